"""CPU ORACLE -- test infrastructure, not product code.

ctypes front end of ``winograd_oracle.c`` and ``winograd_f2x2_oracle.c`` (plain C, built with gcc).  Only
tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the HIP library and its Python binding never do, and nothing here
imports them.  Arrays are numpy; activations and outputs are NCHW, filters
[K][C][3][3]; NHWC callers transpose with numpy before and after.

Transformed tiles are returned as int64 arrays whose last three axes are
[6][6][2] = (row, column, (re, im)) of the full complex 6x6 tile: conjugate
symmetry (Section 3.4 of the paper) is never used to fill entries in.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "winograd_oracle.c"), os.path.join(_HERE, "winograd_f2x2_oracle.c")]
_LIB = os.path.join(_HERE, "liboracle.so")


_CHECK_SRC = os.path.join(_HERE, "sanitize_check.c")
_CHECK_BIN = os.path.join(_HERE, "sanitize_check")


def build(force=False, sanitize=False):
    """Compile the oracle with gcc -O2 (OpenMP over the outermost loops only).  sanitize=True builds instead the
    self-checking program sanitize_check.c together with the oracle's sources under AddressSanitizer and
    UndefinedBehaviorSanitizer (any finding aborts the program) and returns its path."""
    if sanitize:
        srcs = _SRCS + [_CHECK_SRC]
        if force or not os.path.exists(_CHECK_BIN) or os.path.getmtime(_CHECK_BIN) < max(os.path.getmtime(s) for s in srcs):
            subprocess.check_call(
                ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-Wall", "-fsanitize=address,undefined",
                 "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-o", _CHECK_BIN] + srcs + ["-lm"])
        return _CHECK_BIN
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(s) for s in _SRCS):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", _LIB] + _SRCS
        )
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_scale_round.restype = ctypes.c_int64
        _lib.oracle_scale_round.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i8(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.int8, a.dtype
    return a


def num_threads():
    return int(lib().oracle_num_threads())


def matrices():
    """(B^T [6,6], G' = 4G [6,3], A^T [4,6]) as complex128 arrays (Section 3.3)."""
    bt = np.zeros((6, 6, 2), np.int8)
    g4 = np.zeros((6, 3, 2), np.int8)
    at = np.zeros((4, 6, 2), np.int8)
    lib().oracle_get_matrices(_p(bt), _p(g4), _p(at))
    cx = lambda m: m[..., 0].astype(np.float64) + 1j * m[..., 1].astype(np.float64)
    return cx(bt), cx(g4), cx(at)


def partner_map():
    """[6,6,2]: (r', c') with X[r,c] = conj(X[r',c']); self-partnered, real-row/col = real."""
    out = np.zeros((6, 6, 2), np.int32)
    lib().oracle_partner_map(_p(out))
    return out


def direct_conv2d(x, g):
    """Direct 3x3 stride-1 pad-1 correlation, int64 accumulate -> int32 (Section 3.2)."""
    x, g = _i8(x), _i8(g)
    N, C, H, W = x.shape
    K = g.shape[0]
    assert g.shape == (K, C, 3, 3)
    y = np.zeros((N, K, H, W), np.int32)
    ovf = lib().oracle_direct_conv2d(_p(x), _p(g), _p(y), N, C, H, W, K)
    if ovf:
        raise OverflowError("direct convolution does not fit int32")
    return y


def f43_1d(d, g):
    """1-D F(4,3) with G' = 4G: complex int64 [4] = 4 * FIR(d, g)."""
    d = np.ascontiguousarray(d, np.int64)
    g = np.ascontiguousarray(g, np.int64)
    re = np.zeros(4, np.int64)
    im = np.zeros(4, np.int64)
    lib().oracle_f43_1d(_p(d), _p(g), _p(re), _p(im))
    return re, im


def tiles(N, H, W):
    return N * ((H + 3) // 4) * ((W + 3) // 4)


def input_transform(x):
    """D = B^T d B for every tile/channel: int64 [T, C, 6, 6, 2]."""
    x = _i8(x)
    N, C, H, W = x.shape
    out = np.zeros((tiles(N, H, W), C, 6, 6, 2), np.int64)
    lib().oracle_input_transform(_p(x), N, C, H, W, _p(out))
    return out


def filter_transform(g):
    """W = G' g G'^T: int64 [K, C, 6, 6, 2]."""
    g = _i8(g)
    K, C = g.shape[:2]
    out = np.zeros((K, C, 6, 6, 2), np.int64)
    lib().oracle_filter_transform(_p(g), K, C, _p(out))
    return out


def contract(D, Wt):
    """M[t,k] = sum_c W[k,c] (.) D[t,c]: int64 [T, K, 6, 6, 2]."""
    D = np.ascontiguousarray(D, np.int64)
    Wt = np.ascontiguousarray(Wt, np.int64)
    T, C = D.shape[:2]
    K = Wt.shape[0]
    assert Wt.shape[1] == C
    M = np.zeros((T, K, 6, 6, 2), np.int64)
    lib().oracle_contract(_p(D), _p(Wt), ctypes.c_int64(T), C, K, _p(M))
    return M


def output_transform(M, N, K, H, W, shift=4, round_add=0):
    """((A^T M A) + round_add) >> shift, NCHW int32; also returns the flag mask."""
    M = np.ascontiguousarray(M, np.int64)
    assert M.shape == (tiles(N, H, W), K, 6, 6, 2)
    y = np.zeros((N, K, H, W), np.int32)
    flags = lib().oracle_output_transform(_p(M), N, K, H, W, shift, ctypes.c_int64(round_add), _p(y))
    return y, int(flags)


def worstcase_magnitude(Gm, gpos, gneg):
    """Worst-case |Re|, |Im| of every entry of G' g G'^T for taps in [-gneg, gpos] (Section 4.1)."""
    Gm = np.asarray(Gm)
    rows = Gm.shape[0]
    packed = np.zeros((rows, 3, 2), np.int32)
    packed[..., 0] = np.real(Gm).astype(np.int32)
    packed[..., 1] = np.imag(Gm).astype(np.int32)
    re = np.zeros((rows, rows), np.int64)
    im = np.zeros((rows, rows), np.int64)
    lib().oracle_worstcase_magnitude(_p(packed), rows, ctypes.c_int64(gpos), ctypes.c_int64(gneg), _p(re), _p(im))
    return re, im


def worstcase_input_magnitude(dpos, dneg):
    re = np.zeros((6, 6), np.int64)
    im = np.zeros((6, 6), np.int64)
    lib().oracle_worstcase_input_magnitude(ctypes.c_int64(dpos), ctypes.c_int64(dneg), _p(re), _p(im))
    return re, im


def scale_factor(mx, weight_range):
    """(n, p): down-scale factor n / 2^p of Section 4.2; (0, 0) = no scaling."""
    n = ctypes.c_int32()
    p = ctypes.c_int32()
    lib().oracle_scale_factor(ctypes.c_int64(int(mx)), ctypes.c_int64(int(weight_range)), ctypes.byref(n), ctypes.byref(p))
    return n.value, p.value


def inverse_factor(n, p):
    """(r, q): 8-bit multiplier and shift approximating 2^p / n (Section 4.2)."""
    r = ctypes.c_int32()
    q = ctypes.c_int32()
    lib().oracle_inverse_factor(int(n), int(p), ctypes.byref(r), ctypes.byref(q))
    return r.value, q.value


def scale_round(v, mul, sh):
    return int(lib().oracle_scale_round(int(v), int(mul), int(sh)))


def scale_filters(Wt, weight_range):
    """Down-scale Winograd-domain filters per (k, location).  Returns (W~, tab[K,6,6,4], mx[K,6,6])."""
    Wt = np.array(Wt, dtype=np.int64, order="C", copy=True)
    K, C = Wt.shape[:2]
    tab = np.zeros((K, 6, 6, 4), np.int32)
    mx = np.zeros((K, 6, 6), np.int64)
    lib().oracle_scale_filters(_p(Wt), K, C, ctypes.c_int64(weight_range), _p(tab), _p(mx))
    return Wt, tab, mx


def inverse_scale(M, tab):
    M = np.array(M, dtype=np.int64, order="C", copy=True)
    T, K = M.shape[:2]
    tab = np.ascontiguousarray(tab, np.int32)
    lib().oracle_inverse_scale(_p(M), ctypes.c_int64(T), K, _p(tab))
    return M


def scale_activations(D, value_range=127):
    """The rule of Section 4.2 applied per tile to [T,C,6,6,2] transformed activations: (scaled copy, table
    [T,6,6,4] = (n,p,r,q), max [T,6,6])."""
    D = np.array(D, dtype=np.int64, order="C", copy=True)
    T, C = D.shape[:2]
    tab = np.zeros((T, 6, 6, 4), np.int32)
    mx = np.zeros((T, 6, 6), np.int64)
    lib().oracle_scale_activations(_p(D), ctypes.c_int64(T), C, ctypes.c_int64(value_range), _p(tab), _p(mx))
    return D, tab, mx


def inverse_scale_tiles(M, atab):
    M = np.array(M, dtype=np.int64, order="C", copy=True)
    T, K = M.shape[:2]
    atab = np.ascontiguousarray(atab, np.int32)
    lib().oracle_inverse_scale_tiles(_p(M), ctypes.c_int64(T), K, _p(atab))
    return M


LOSSLESS, SCALED = 0, 1


def winograd_conv2d(x, g, mode=LOSSLESS, weight_range=127):
    """Whole complex-Winograd path.  Returns (y int32 NCHW, flags)."""
    x, g = _i8(x), _i8(g)
    N, C, H, W = x.shape
    K = g.shape[0]
    assert g.shape == (K, C, 3, 3)
    y = np.zeros((N, K, H, W), np.int32)
    flags = lib().oracle_winograd_conv2d(_p(x), _p(g), _p(y), N, C, H, W, K, mode, ctypes.c_int64(weight_range))
    if flags < 0:
        raise MemoryError("oracle ran out of memory")
    return y, int(flags)


def requant_relu_pool(y, shift, relu=True, pool=False):
    y = np.ascontiguousarray(y, np.int32)
    N, K, H, W = y.shape
    if pool:
        assert H % 2 == 0 and W % 2 == 0
    out = np.zeros((N, K, H // 2 if pool else H, W // 2 if pool else W), np.int8)
    lib().oracle_requant_relu_pool(_p(y), _p(out), N, K, H, W, shift, int(relu), int(pool))
    return out


# ---- rational F(2x2,3x3) in integers (the running example of Sections 4.1-4.2) --------------------------------

def f2_matrices():
    """(B^T [4,4], G' = 2G [4,3], A^T [2,4]) as int64 arrays."""
    bt, g2, at = np.zeros((4, 4), np.int8), np.zeros((4, 3), np.int8), np.zeros((2, 4), np.int8)
    lib().oracle_f2_get_matrices(_p(bt), _p(g2), _p(at))
    return bt.astype(np.int64), g2.astype(np.int64), at.astype(np.int64)


def f2_filter_transform(g):
    """G' g G'^T for [K,C,3,3] int8 filters -> int64 [K,C,4,4]."""
    g = _i8(g)
    K, C = g.shape[:2]
    out = np.zeros((K, C, 4, 4), np.int64)
    lib().oracle_f2_filter_transform(_p(g), K, C, _p(out))
    return out


def f2_input_transform(x):
    """B^T d B for every 4x4 input tile (stride 2, pad 1) -> int64 [T,C,4,4], T = N*ceil(H/2)*ceil(W/2)."""
    x = _i8(x)
    N, C, H, W = x.shape
    out = np.zeros((N * ((H + 1) // 2) * ((W + 1) // 2), C, 4, 4), np.int64)
    lib().oracle_f2_input_transform(_p(x), N, C, H, W, _p(out))
    return out


def f2_scale_filters(Wt, weight_range=127):
    """Section 4.2 on [K,C,4,4] Winograd-domain filters: (scaled copy, table [K,4,4,4] = (n,p,r,q), max [K,4,4])."""
    Wt = np.ascontiguousarray(Wt, dtype=np.int64).copy()
    K, C = Wt.shape[:2]
    tab = np.zeros((K, 4, 4, 4), np.int32)
    mx = np.zeros((K, 4, 4), np.int64)
    lib().oracle_f2_scale_filters(_p(Wt), K, C, ctypes.c_int64(weight_range), _p(tab), _p(mx))
    return Wt, tab, mx


BOTH_SCALED = 2   # filters and activations scaled (signed int8 data)


def f2_scale_activations(D, value_range=127):
    """The rule of Section 4.2 applied per tile to [T,C,4,4] transformed activations: (scaled copy, table [T,4,4,4] =
    (n,p,r,q), max [T,4,4])."""
    D = np.ascontiguousarray(D, dtype=np.int64).copy()
    T, C = D.shape[:2]
    tab = np.zeros((T, 4, 4, 4), np.int32)
    mx = np.zeros((T, 4, 4), np.int64)
    lib().oracle_f2_scale_activations(_p(D), ctypes.c_int64(T), C, ctypes.c_int64(value_range), _p(tab), _p(mx))
    return D, tab, mx


def f2_conv2d(x, g, mode=LOSSLESS, weight_range=127):
    """Whole F(2x2,3x3) path.  Returns (y int32 NCHW, flags)."""
    x, g = _i8(x), _i8(g)
    N, C, H, W = x.shape
    K = g.shape[0]
    assert g.shape == (K, C, 3, 3)
    y = np.zeros((N, K, H, W), np.int32)
    flags = lib().oracle_f2_conv2d(_p(x), _p(g), _p(y), N, C, H, W, K, mode, ctypes.c_int64(weight_range))
    if flags < 0:
        raise MemoryError("oracle ran out of memory")
    return y, int(flags)


def _i16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.int16, a.dtype
    return a


def direct_conv2d_i16(x, g):
    """Direct 3x3 stride-1 pad-1 correlation of int16 arrays (e.g. uint8 minus zero point) -> int32 NCHW."""
    x, g = _i16(x), _i16(g)
    N, C, H, W = x.shape
    K = g.shape[0]
    assert g.shape == (K, C, 3, 3)
    y = np.zeros((N, K, H, W), np.int32)
    flags = lib().oracle_direct_conv2d_i16(_p(x), _p(g), _p(y), N, C, H, W, K)
    assert flags == 0, "output does not fit int32"
    return y


def input_transform_i16(x):
    """D = B^T d B of int16 (int9) activations: int64 [T, C, 6, 6, 2]."""
    x = _i16(x)
    N, C, H, W = x.shape
    out = np.zeros((tiles(N, H, W), C, 6, 6, 2), np.int64)
    lib().oracle_input_transform_i16(_p(x), N, C, H, W, _p(out))
    return out


def filter_transform_i16(g):
    """W = G' g G'^T of int16 (int9) filters: int64 [K, C, 6, 6, 2]."""
    g = _i16(g)
    K, C = g.shape[:2]
    out = np.zeros((K, C, 6, 6, 2), np.int64)
    lib().oracle_filter_transform_i16(_p(g), K, C, _p(out))
    return out


def winograd_conv2d_i16(x, g, mode=LOSSLESS, weight_range=127):
    """Whole complex-Winograd path on int16 inputs (int9 values).  Returns (y int32 NCHW, flags)."""
    x, g = _i16(x), _i16(g)
    N, C, H, W = x.shape
    K = g.shape[0]
    assert g.shape == (K, C, 3, 3)
    y = np.zeros((N, K, H, W), np.int32)
    flags = lib().oracle_winograd_conv2d_i16(_p(x), _p(g), _p(y), N, C, H, W, K, mode, ctypes.c_int64(weight_range))
    if flags < 0:
        raise MemoryError("oracle ran out of memory")
    return y, int(flags)


def f2_filter_transform_i16(g):
    g = _i16(g)
    K, C = g.shape[:2]
    out = np.zeros((K, C, 4, 4), np.int64)
    lib().oracle_f2_filter_transform_i16(_p(g), K, C, _p(out))
    return out


def f2_conv2d_i16(x, g, mode=LOSSLESS, weight_range=127):
    """F(2x2,3x3) path on int16 inputs (int9 values).  Returns (y int32 NCHW, flags)."""
    x, g = _i16(x), _i16(g)
    N, C, H, W = x.shape
    K = g.shape[0]
    assert g.shape == (K, C, 3, 3)
    y = np.zeros((N, K, H, W), np.int32)
    flags = lib().oracle_f2_conv2d_i16(_p(x), _p(g), _p(y), N, C, H, W, K, mode, ctypes.c_int64(weight_range))
    if flags < 0:
        raise MemoryError("oracle ran out of memory")
    return y, int(flags)
