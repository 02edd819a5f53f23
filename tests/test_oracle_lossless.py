"""Pins for the CPU oracle's lossless path: the direct convolution, the three
transforms, the conjugate structure and the exact identity Winograd == direct.

Nothing here touches the GPU.  Each pin is chosen so that a plausible slip in
the oracle (a wrong sign or index in a matrix, a transposed operand, a flipped
kernel, a wrong tile origin) fails at least one of them.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
from tests import golden_io
from paper_1901_01965_amd import workloads as wl


# ----------------------------------------------------------------------------
# the printed matrices (Section 3.3)

def test_matrices_are_the_printed_ones():
    gold = golden_io.sections("complex_f4x4_3x3_matrices.txt")
    bt, g4, at = oracle.matrices()
    assert np.array_equal(bt, gold["BT"])
    assert np.array_equal(g4, 4 * gold["G"])          # the oracle holds G' = 4 G
    assert np.array_equal(at, gold["AT"])


def test_matrices_interpolate_the_stated_points():
    """Rows 0..4 of each printed matrix belong to the points 0, 1, -1, i, -i (Section 3.3):
    G evaluates the filter polynomial there (up to the row's constant), A^T holds the
    powers of the points.  A fixture typo would break this structure."""
    gold = golden_io.sections("complex_f4x4_3x3_matrices.txt")
    pts = np.array([0, 1, -1, 1j, -1j])
    G, AT = gold["G"], gold["AT"]
    for r, p in enumerate(pts):
        vander = np.array([1, p, p * p])
        ratio = G[r] / vander if p != 0 else None
        if p == 0:
            assert np.array_equal(G[r], [1, 0, 0])
        else:
            assert np.allclose(ratio, ratio[0])          # G[r] is proportional to (1, p, p^2)
        assert np.allclose(AT[:, r], [1, p, p ** 2, p ** 3])
    assert np.array_equal(G[5], [0, 0, 1])                # the point at infinity
    assert np.array_equal(AT[:, 5], [0, 0, 0, 1])


# ----------------------------------------------------------------------------
# direct convolution

@pytest.mark.parametrize("shape", [(1, 1, 1, 1, 1), (2, 3, 5, 7, 4), (1, 4, 9, 6, 3), (3, 2, 4, 4, 5)])
def test_direct_matches_library_conv2d(shape):
    N, C, H, W, K = shape
    x, g = wl.make_custom(N, C, K, H, W, seed=1)
    want = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(g).double(), padding=1)
    assert np.array_equal(oracle.direct_conv2d(x, g), want.numpy().astype(np.int64))


def test_direct_is_correlation_not_flipped():
    """A single tap at filter position (a, b) shifts the image by (a-1, b-1): y[h,w] = x[h+a-1, w+b-1]."""
    x, _ = wl.make_custom(1, 1, 1, 6, 5, seed=2)
    for a, b in itertools.product(range(3), range(3)):
        g = np.zeros((1, 1, 3, 3), np.int8)
        g[0, 0, a, b] = 1
        y = oracle.direct_conv2d(x, g)[0, 0]
        pad = np.pad(x[0, 0].astype(np.int32), 1)
        assert np.array_equal(y, pad[a:a + 6, b:b + 5])


def test_direct_brute_force_python_loops():
    x, g = wl.make_custom(1, 2, 2, 3, 4, seed=3)
    y = oracle.direct_conv2d(x, g)
    for k, h, w in itertools.product(range(2), range(3), range(4)):
        s = 0
        for c, a, b in itertools.product(range(2), range(3), range(3)):
            hh, ww = h + a - 1, w + b - 1
            if 0 <= hh < 3 and 0 <= ww < 4:
                s += int(x[0, c, hh, ww]) * int(g[k, c, a, b])
        assert y[0, k, h, w] == s


def test_direct_overflow_is_reported():
    x = np.full((1, 1024, 3, 3), -128, np.int8)
    g = np.full((32, 1024, 3, 3), -128, np.int8)
    # 9 * 1024 * 16384 = 150994944 < 2^31, still fits
    oracle.direct_conv2d(x[:, :1024], g[:1])
    big_x = np.full((1, 16384, 3, 3), -128, np.int8)
    big_g = np.full((1, 16384, 3, 3), -128, np.int8)
    with pytest.raises(OverflowError):
        oracle.direct_conv2d(big_x, big_g)


# ----------------------------------------------------------------------------
# one-dimensional F(4,3) (Section 3.2)

def test_f43_1d_is_four_times_the_fir_filter():
    rng = np.random.default_rng(5)
    for _ in range(50):
        d = rng.integers(-128, 128, 6)
        g = rng.integers(-128, 128, 3)
        re, im = oracle.f43_1d(d, g)
        fir = np.array([sum(g[j] * d[k + j] for j in range(3)) for k in range(4)])
        assert np.array_equal(re, 4 * fir)
        assert not im.any()


# ----------------------------------------------------------------------------
# transforms against plain matrix products with the printed matrices

def _tiles_numpy(x):
    """[T, C, 6, 6] input tiles (stride 4, origin -1, zero padded), by slicing a padded copy."""
    N, C, H, W = x.shape
    TH, TW = (H + 3) // 4, (W + 3) // 4
    pad = np.zeros((N, C, 4 * TH + 2, 4 * TW + 2), np.int64)
    pad[:, :, 1:H + 1, 1:W + 1] = x
    out = np.zeros((N, TH, TW, C, 6, 6), np.int64)
    for ty in range(TH):
        for tx in range(TW):
            out[:, ty, tx] = pad[:, :, 4 * ty:4 * ty + 6, 4 * tx:4 * tx + 6]
    return out.reshape(N * TH * TW, C, 6, 6)


def _cx(a):
    return a[..., 0] + 1j * a[..., 1]


@pytest.mark.parametrize("hw", [(4, 4), (8, 12), (7, 5), (1, 1), (9, 2)])
def test_input_transform_is_BT_d_B(hw):
    gold = golden_io.sections("complex_f4x4_3x3_matrices.txt")
    BT = gold["BT"]
    x, _ = wl.make_custom(2, 3, 1, hw[0], hw[1], seed=7)
    D = _cx(oracle.input_transform(x))
    d = _tiles_numpy(x)
    want = np.einsum("ra,tcab,sb->tcrs", BT, d, BT)       # B = (B^T)^T, plain transpose
    assert np.array_equal(D, want)


def test_input_transform_row_expansion():
    """The expansion of d' = B^T d printed at the start of Section 3.4, checked through a
    tile that is zero except in one column (so that D[:, 0] = d'[:, 0] - d'[:, 4] isolates it)."""
    x = np.zeros((1, 1, 4, 4), np.int8)
    col = np.array([0, 5, -7, 11, 13, 0])                 # rows -1..4 of the padded tile, column 0
    x[0, 0, :, 0] = col[1:5]                              # column w=0 is tile column 1
    D = _cx(oracle.input_transform(x))[0, 0]              # single tile
    d = col
    dprime = np.array([
        d[0] - d[4],
        d[1] + d[2] + d[3] + d[4],
        -d[1] + d[2] - d[3] + d[4],
        -d[2] + d[4] - (d[1] - d[3]) * 1j,
        -d[2] + d[4] + (d[1] - d[3]) * 1j,
        -d[1] + d[5],
    ])
    # tile column 1 holds the data; D[:, 5] = d'[:, 5] - d'[:, 1] = -d'[:, 1]
    assert np.array_equal(D[:, 5], -dprime)


def test_filter_transform_is_G_g_GT():
    gold = golden_io.sections("complex_f4x4_3x3_matrices.txt")
    G4 = 4 * gold["G"]
    _, g = wl.make_custom(1, 3, 4, 4, 4, seed=8)
    Wt = _cx(oracle.filter_transform(g))
    want = np.einsum("ra,kcab,sb->kcrs", G4, g.astype(np.int64), G4)
    assert np.array_equal(Wt, want)


# ----------------------------------------------------------------------------
# conjugate structure (Section 3.4)

def _check_pattern(X):
    """X: complex [..., 6, 6] must follow the printed pattern exactly."""
    pat = golden_io.conjugate_pattern()
    for r in range(6):
        for c in range(6):
            pr, pc, conj = pat[r][c]
            ref = X[..., pr, pc]
            assert np.array_equal(X[..., r, c], np.conj(ref) if conj else ref), (r, c)
    real_rc = [0, 1, 2, 5]
    for r in real_rc:
        for c in real_rc:
            assert not np.imag(X[..., r, c]).any(), (r, c)


def test_conjugate_pattern_of_D_W_and_M():
    x, g = wl.make_custom(1, 3, 2, 8, 8, seed=9)
    D = oracle.input_transform(x)
    Wt = oracle.filter_transform(g)
    M = oracle.contract(D, Wt)
    _check_pattern(_cx(D))
    _check_pattern(_cx(Wt))
    _check_pattern(_cx(M))


def test_partner_map_matches_printed_pattern_and_counts():
    pat = golden_io.conjugate_pattern()
    pm = oracle.partner_map()
    const = golden_io.constants()
    pairs, reals, complex_free = 0, 0, 0
    for r in range(6):
        for c in range(6):
            pr, pc, conj = pat[r][c]
            assert (pm[r, c, 0], pm[r, c, 1]) == (pr, pc)
            assert conj == ((pr, pc) != (r, c))
            if conj:
                pairs += 1
            elif r in (0, 1, 2, 5) and c in (0, 1, 2, 5):
                reals += 1
            else:
                complex_free += 1
    assert reals == const["real_entries"]
    assert pairs == complex_free == const["conjugate_pairs"]
    mults = reals + 3 * pairs                              # three real products per complex one
    assert mults == const["general_mults_complex_f4x4_3x3"]
    assert round(const["general_mults_direct"] / mults, 2) == const["complexity_reduction"]


# ----------------------------------------------------------------------------
# lossless Winograd == direct, exactly

SHAPES = [
    # N, C, K, H, W
    (1, 1, 1, 4, 4), (1, 1, 1, 1, 1), (1, 3, 1, 2, 3), (2, 1, 3, 5, 5), (1, 3, 3, 7, 9),
    (1, 2, 2, 8, 8), (1, 2, 2, 6, 4), (2, 3, 3, 9, 1), (1, 5, 4, 13, 10),
]


@pytest.mark.parametrize("shape", SHAPES)
def test_lossless_winograd_equals_direct(shape):
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, seed=11)
    y, flags = oracle.winograd_conv2d(x, g, oracle.LOSSLESS)
    assert flags == 0          # imaginary parts vanish and A^T M A is a multiple of 16
    assert np.array_equal(y, oracle.direct_conv2d(x, g))


@pytest.mark.parametrize("xv,gv", [(-128, -128), (127, -128), (-128, 127), (127, 127)])
def test_lossless_at_the_int8_extremes(xv, gv):
    x = np.full((1, 2, 8, 8), xv, np.int8)
    g = np.full((2, 2, 3, 3), gv, np.int8)
    y, flags = oracle.winograd_conv2d(x, g, oracle.LOSSLESS)
    assert flags == 0
    assert np.array_equal(y, oracle.direct_conv2d(x, g))


def test_lossless_checkerboard_extremes():
    """Alternating +-extremes drive the mixed-sign rows of the transforms to their largest values."""
    x = np.where((np.indices((8, 8)).sum(0) % 2) == 0, 127, -128).astype(np.int8)[None, None]
    g = np.where((np.indices((3, 3)).sum(0) % 2) == 0, -128, 127).astype(np.int8)[None, None]
    y, flags = oracle.winograd_conv2d(x, g, oracle.LOSSLESS)
    assert flags == 0
    assert np.array_equal(y, oracle.direct_conv2d(x, g))


def test_delta_filter_is_identity_and_impulse_response_is_filter():
    x, _ = wl.make_custom(1, 1, 1, 8, 8, seed=12)
    g = np.zeros((1, 1, 3, 3), np.int8)
    g[0, 0, 1, 1] = 1
    y, _ = oracle.winograd_conv2d(x, g)
    assert np.array_equal(y[0, 0], x[0, 0])
    imp = np.zeros((1, 1, 8, 8), np.int8)
    imp[0, 0, 4, 3] = 1                                    # sits on a tile boundary row
    _, g = wl.make_custom(1, 1, 1, 8, 8, seed=13)
    y, _ = oracle.winograd_conv2d(imp, g)
    assert np.array_equal(y[0, 0, 3:6, 2:5], g[0, 0, ::-1, ::-1])   # correlation: flipped stamp


def test_stagewise_composition_equals_pipeline():
    x, g = wl.make_custom(2, 3, 2, 7, 6, seed=14)
    D = oracle.input_transform(x)
    Wt = oracle.filter_transform(g)
    M = oracle.contract(D, Wt)
    y, flags = oracle.output_transform(M, 2, 2, 7, 6, shift=4, round_add=0)
    assert flags == 0
    assert np.array_equal(y, oracle.direct_conv2d(x, g))


def test_configuration_one_full_size():
    x, g = wl.make_case("cfg1")
    y, flags = oracle.winograd_conv2d(x, g)
    assert flags == 0
    assert np.array_equal(y, oracle.direct_conv2d(x, g))


def test_requant_relu_pool_against_numpy():
    rng = np.random.default_rng(15)
    y = rng.integers(-5000, 5000, (2, 3, 4, 6)).astype(np.int32)
    for shift in (0, 1, 5):
        for relu in (True, False):
            v = y.astype(np.int64)
            if shift:
                v = (v + (1 << (shift - 1))) >> shift
            v = np.clip(v, 0 if relu else -128, 127)
            assert np.array_equal(oracle.requant_relu_pool(y, shift, relu, False), v.astype(np.int8))
            pooled = v.reshape(2, 3, 2, 2, 3, 2).max(axis=(3, 5))
            assert np.array_equal(oracle.requant_relu_pool(y, shift, relu, True), pooled.astype(np.int8))
