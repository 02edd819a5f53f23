"""Writes tests/golden/vgg16_shifts.txt: the fixed per-layer requantisation shifts of the VGG-16-shaped stack.

Calls only the CPU oracle.  Image 0 of the seeded stack is pushed through the 13 layers with the oracle's
direct convolution; after each layer s = max(0, bitlen(max y) - 7) is frozen, so that activations neither
saturate nor die out, and the layer output is requantised (ReLU, shift, clamp to [0,127], 2x2 max-pool at
stage ends) with the oracle's routine.  Run from the repository root: python tests/golden/make_vgg16_shifts.py
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_1901_01965_amd import workloads as wl  # noqa: E402


def main():
    x, gs = wl.make_vgg16(batch=1)
    shifts = []
    for (cin, cout, hw, pool), g in zip(wl.VGG16_LAYERS, gs):
        y = oracle.direct_conv2d(x, g)
        s = max(0, int(y.max()).bit_length() - 7)
        shifts.append(s)
        x = oracle.requant_relu_pool(y, s, relu=True, pool=pool)
        print("layer %dx%d C=%d K=%d: max y = %d, shift = %d, nonzero after requant = %.1f%%"
              % (hw, hw, cin, cout, y.max(), s, 100.0 * (x != 0).mean()), flush=True)
    out = os.path.join(ROOT, "tests", "golden", "vgg16_shifts.txt")
    with open(out, "w") as f:
        f.write("# Per-layer requantisation shifts of the VGG-16-shaped stack (harness constants, not from the\n")
        f.write("# paper): written by tests/golden/make_vgg16_shifts.py from the CPU oracle on image 0.\n")
        f.write(" ".join(str(s) for s in shifts) + "\n")
    print("wrote", out, shifts)


if __name__ == "__main__":
    main()
