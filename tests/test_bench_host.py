"""Host logic of bench.py that needs no GPU: the refusal of several GPUs, and the per-unit byte and operation counts
the roofline figures are built from (Section 3.4: 46 real products per tile and channel pair; 16 outputs per tile)."""
import os
import subprocess
import sys

import bench
from paper_1901_01965_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert proc.returncode != 0
    assert "one GPU" in proc.stderr and not proc.stdout.strip()


def test_algorithmic_bytes_of_the_quoted_layer():
    case = wl.CASES["cfg2"]
    assert case.tiles == 8 * 14 * 14 and case.direct_ops == 2 * 9 * 8 * 64 * 64 * 56 * 56
    alg = bench.algorithmic_bytes(case, "lossless")
    # 16 B in per (tile, channel), 64 B out per (tile, filter), the lossless filters (26 entries as 72 int8 planes) once
    assert alg["fused_conv"] == 16 * 1568 * 64 + 64 * 1568 * 64 + 72 * 64 * 64 == 8_323_072
    assert alg["input_transform"] == (16 + 72) * 1568 * 64
    assert alg["output_transform"] == (144 + 64) * 1568 * 64
    lay = bench.layout_bytes(case, "lossless")
    assert lay["fused_conv"] - alg["fused_conv"] == (138 - 72) * 64 * 64      # the three-operand lossless filter planes
    assert all(lay[k] >= alg[k] for k in alg)


def test_matrix_core_work_counts_the_methods_products():
    case = wl.CASES["cfg2"]
    pairs = case.tiles * case.C * case.K
    assert bench.contraction_int8_ops(case, "lossless") == 2 * 46 * 3 * pairs       # 46 products x three limb products
    assert bench.contraction_int8_ops(case, "scaled") == 2 * 112 * pairs
    # the direct method multiplies 144 times per tile and channel pair (16 outputs x 9 taps)
    assert case.direct_ops == 2 * 144 * pairs
