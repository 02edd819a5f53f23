"""Seeded synthetic inputs for the 3x3 convolution workloads.

This module only makes numbers: it holds none of the Winograd arithmetic and is
the one piece of code that both the HIP tests/benchmark and the CPU oracle's
tests are fed from.  All tensors are numpy, activations NCHW int8 and filters
[K][C][3][3] int8; ``to_nhwc`` / ``to_krsc`` give the channels-last views.

The tensors stand in for the image-classification activations and quantised
weights the paper's own evaluation used (Section 4.4), which are not available
here; only layer shapes and value distributions are reproduced.
"""
from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

BASE_SEED = 190101965


@dataclass(frozen=True)
class ConvCase:
    name: str
    config: int          # 1..5, the workload family
    N: int
    C: int
    K: int
    H: int
    W: int
    act: str             # "uniform" | "relu"
    wgt: str             # "uniform" | "gauss"
    modes: Tuple[str, ...]   # which of ("lossless", "scaled") the workload is run in
    sub: int = 0         # distinguishes tensors of cases in one family

    @property
    def tiles(self):
        return self.N * ((self.H + 3) // 4) * ((self.W + 3) // 4)

    @property
    def direct_ops(self):
        """int8 operations of the direct method: 2 * 9 * N*K*C*H*W."""
        return 2 * 9 * self.N * self.K * self.C * self.H * self.W


CASES = {
    "cfg1": ConvCase("cfg1", 1, 1, 16, 16, 16, 16, "uniform", "uniform", ("lossless",)),
    "cfg2": ConvCase("cfg2", 2, 8, 64, 64, 56, 56, "relu", "gauss", ("lossless",)),
    "cfg3": ConvCase("cfg3", 3, 32, 128, 128, 28, 28, "relu", "gauss", ("lossless", "scaled")),
    "cfg4a": ConvCase("cfg4a", 4, 64, 256, 256, 14, 14, "relu", "gauss", ("scaled",), 0),
    "cfg4b": ConvCase("cfg4b", 4, 64, 512, 512, 7, 7, "relu", "gauss", ("scaled",), 1),
}

# VGG-16-shaped stack: (Cin, Cout, H=W, pool after this layer)
VGG16_LAYERS: List[Tuple[int, int, int, bool]] = [
    (3, 64, 224, False), (64, 64, 224, True),
    (64, 128, 112, False), (128, 128, 112, True),
    (128, 256, 56, False), (256, 256, 56, False), (256, 256, 56, True),
    (256, 512, 28, False), (512, 512, 28, False), (512, 512, 28, True),
    (512, 512, 14, False), (512, 512, 14, False), (512, 512, 14, True),
]
VGG16_BATCH = 16
# Fixed requantisation shifts per layer (harness constants): s = max(0, bitlen(max y) - 7) measured by the CPU
# oracle on image 0, written by tests/golden/make_vgg16_shifts.py into tests/golden/vgg16_shifts.txt.
VGG16_SHIFTS = [9, 9, 9, 10, 10, 10, 10, 11, 10, 10, 11, 11, 10]


def _rng(config, tensor_id):
    return np.random.default_rng(BASE_SEED + 1000 * config + tensor_id)


def activations(kind, shape, rng):
    """int8 NCHW activations.  "uniform": all of [-128,127]; "relu": half zeros, rest uniform [0,127]."""
    if kind == "uniform":
        return rng.integers(-128, 128, size=shape, dtype=np.int8)
    if kind == "relu":
        vals = rng.integers(0, 128, size=shape, dtype=np.int16)
        zero = rng.random(size=shape) < 0.5
        return np.where(zero, 0, vals).astype(np.int8)
    raise ValueError(kind)


def weights(kind, shape, rng):
    """int8 [K,C,3,3] filters.  "uniform": [-128,127]; "gauss": round(N(0, sigma=32)) clipped to [-127,127]."""
    if kind == "uniform":
        return rng.integers(-128, 128, size=shape, dtype=np.int8)
    if kind == "gauss":
        return np.clip(np.rint(rng.normal(0.0, 32.0, size=shape)), -127, 127).astype(np.int8)
    raise ValueError(kind)


def make_case(case, batch=None):
    """(x [N,C,H,W] int8, g [K,C,3,3] int8) for a ConvCase; ``batch`` overrides N (prefix-stable)."""
    if isinstance(case, str):
        case = CASES[case]
    N = case.N if batch is None else batch
    x = np.concatenate(
        [activations(case.act, (1, case.C, case.H, case.W), _rng(case.config, 100 * case.sub + 10 + n))
         for n in range(N)], axis=0)
    g = weights(case.wgt, (case.K, case.C, 3, 3), _rng(case.config, 100 * case.sub + 1))
    return x, g


def make_custom(N, C, K, H, W, act="uniform", wgt="uniform", seed=0):
    """Free-form case for edge-case tests (ragged tiles, odd channel counts, ...)."""
    rng = np.random.default_rng(BASE_SEED + 7919 * seed + 31 * (N + 3 * C + 5 * K + 7 * H + 11 * W))
    return activations(act, (N, C, H, W), rng), weights(wgt, (K, C, 3, 3), rng)


def make_vgg16(batch=VGG16_BATCH):
    """Layer-0 input [batch,3,224,224] and the 13 filters of the VGG-16-shaped stack."""
    x = np.concatenate([activations("relu", (1, 3, 224, 224), _rng(5, 10 + n)) for n in range(batch)], axis=0)
    gs = [weights("gauss", (cout, cin, 3, 3), _rng(5, 1000 + i)) for i, (cin, cout, _, _) in enumerate(VGG16_LAYERS)]
    return x, gs


def to_nhwc(x):
    return np.ascontiguousarray(np.transpose(x, (0, 2, 3, 1)))


def from_nhwc(x):
    return np.ascontiguousarray(np.transpose(x, (0, 3, 1, 2)))


def to_krsc(g):
    return np.ascontiguousarray(np.transpose(g, (0, 2, 3, 1)))
