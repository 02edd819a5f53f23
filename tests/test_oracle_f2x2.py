"""Pins for the CPU oracle's rational F(2x2,3x3) integer path (the running example of Sections 4.1-4.2).  No GPU.

The general lossy result of its scaled mode has no printed worked example: PARITY UNPINNED beyond the special
cases checked here.
"""
import itertools

import numpy as np
import pytest

import oracle
from tests import golden_io
from paper_1901_01965_amd import workloads as wl


def test_filter_matrix_is_the_printed_one():
    gold = golden_io.sections("f2x2_3x3_worstcase.txt")
    _, g2, _ = oracle.f2_matrices()
    assert np.array_equal(g2, np.real(gold["GP"]).astype(np.int64))


def test_filter_transform_matches_the_printed_expansion():
    """Section 4.1 prints G' g row by row and G' g G'^T in terms of its entries p_0..p_11 (row-major)."""
    rng = np.random.default_rng(1)
    g = rng.integers(-128, 128, (5, 3, 3, 3), dtype=np.int8)
    Wt = oracle.f2_filter_transform(g)
    for k in range(5):
        for c in range(3):
            f = g[k, c].astype(np.int64)
            p = np.array([2 * f[0], f[0] + f[1] + f[2], f[0] - f[1] + f[2], 2 * f[2]]).reshape(-1)   # p_0..p_11
            want = np.array([[2 * p[3 * r], p[3 * r] + p[3 * r + 1] + p[3 * r + 2], p[3 * r] - p[3 * r + 1] + p[3 * r + 2],
                              2 * p[3 * r + 2]] for r in range(4)])
            assert np.array_equal(Wt[k, c], want)


def test_filter_transform_reaches_the_printed_worst_case_for_int8():
    """The corners of the int8 box drive G' g G'^T to the magnitudes of the routine that is pinned to the printed
    int9 table; for int8 they need 12 bits."""
    gold = golden_io.sections("f2x2_3x3_worstcase.txt")
    corners = np.array(list(itertools.product([-128, 127], repeat=9)), np.int8).reshape(-1, 1, 3, 3)
    Wt = oracle.f2_filter_transform(corners)
    re, _ = oracle.worstcase_magnitude(gold["GP"], 127, 128)
    assert np.array_equal(np.abs(Wt).max(axis=(0, 1)), re)
    assert int(np.abs(Wt).max()) == 9 * 128


def test_one_dimensional_f23_against_brute_force():
    """A^T [(G' g) (.) (B^T d)] = 2 x the two outputs of the 3-tap correlation of four inputs."""
    bt, g2, at = oracle.f2_matrices()
    rng = np.random.default_rng(2)
    for _ in range(200):
        d = rng.integers(-128, 128, 4)
        g = rng.integers(-128, 128, 3)
        got = at @ ((g2 @ g) * (bt @ d))
        want = 2 * np.array([d[0] * g[0] + d[1] * g[1] + d[2] * g[2], d[1] * g[0] + d[2] * g[1] + d[3] * g[2]])
        assert np.array_equal(got, want)


def test_input_transform_is_bt_d_b_on_padded_tiles():
    bt, _, _ = oracle.f2_matrices()
    x, _ = wl.make_custom(2, 3, 1, 5, 7, seed=3)
    D = oracle.f2_input_transform(x)
    xp = np.pad(x.astype(np.int64), ((0, 0), (0, 0), (1, 2), (1, 2)))
    TH, TW = 3, 4
    assert D.shape == (2 * TH * TW, 3, 4, 4)
    for n in range(2):
        for ty in range(TH):
            for tx in range(TW):
                for c in range(3):
                    d = xp[n, c, 2 * ty:2 * ty + 4, 2 * tx:2 * tx + 4]
                    assert np.array_equal(D[(n * TH + ty) * TW + tx, c], bt @ d @ bt.T)


@pytest.mark.parametrize("shape", [(1, 1, 1, 1, 1), (1, 2, 3, 2, 2), (2, 3, 4, 5, 7), (1, 5, 2, 8, 6), (1, 4, 4, 3, 9)])
def test_lossless_equals_direct_convolution(shape):
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, seed=4)
    y, flags = oracle.f2_conv2d(x, g, oracle.LOSSLESS)
    assert flags == 0          # in particular: every A^T M A was divisible by 4
    assert np.array_equal(y, oracle.direct_conv2d(x, g))


def test_lossless_extreme_values():
    for xv, gv in ((-128, -128), (127, -128), (-128, 127)):
        x = np.full((1, 3, 4, 6), xv, np.int8)
        g = np.full((2, 3, 3, 3), gv, np.int8)
        y, flags = oracle.f2_conv2d(x, g, oracle.LOSSLESS)
        assert flags == 0 and np.array_equal(y, oracle.direct_conv2d(x, g))


def test_scaled_filters_fit_the_range_and_table_comes_from_the_pinned_routines():
    _, g = wl.make_custom(1, 24, 6, 4, 4, wgt="uniform", seed=5)
    Wt = oracle.f2_filter_transform(g)
    for rng_ in (127, 255):
        scaled, tab, mx = oracle.f2_scale_filters(Wt, rng_)
        assert np.array_equal(mx, np.abs(Wt).max(axis=1))
        assert np.abs(scaled).max() <= rng_
        for k in range(6):
            for r in range(4):
                for c in range(4):
                    n, p = oracle.scale_factor(int(mx[k, r, c]), rng_)
                    rr, q = oracle.inverse_factor(n, p)
                    assert tuple(tab[k, r, c]) == (n, p, rr, q)
                    if n == 0:
                        assert np.array_equal(scaled[k, :, r, c], Wt[k, :, r, c])
                    else:   # round half up of w * n / 2^p
                        want = (Wt[k, :, r, c] * n + (1 << (p - 1))) >> p
                        assert np.array_equal(scaled[k, :, r, c], want)
    assert (tab[..., 0] != 0).mean() > 0.5       # uniform int8 filters: most locations exceed 127


def test_scaled_equals_lossless_when_no_location_needs_scaling():
    x, _ = wl.make_custom(1, 6, 3, 6, 6, seed=6)
    g = np.random.default_rng(7).integers(-3, 4, (3, 6, 3, 3)).astype(np.int8)   # 9 * 3 * ... stays below 127
    assert np.abs(oracle.f2_filter_transform(g)).max() <= 127
    y, flags = oracle.f2_conv2d(x, g, oracle.SCALED, 127)
    assert (flags & 4) == 0 and np.array_equal(y, oracle.direct_conv2d(x, g))
    # and with a range that nothing exceeds, any filters
    x, g = wl.make_custom(1, 6, 3, 6, 6, seed=8)
    y, _ = oracle.f2_conv2d(x, g, oracle.SCALED, 1 << 20)
    assert np.array_equal(y, oracle.direct_conv2d(x, g))


def test_scaled_error_is_small_relative_to_signal():
    x, g = wl.make_custom(2, 32, 8, 12, 12, act="relu", wgt="gauss", seed=9)
    want = oracle.direct_conv2d(x, g).astype(np.int64)
    y, flags = oracle.f2_conv2d(x, g, oracle.SCALED, 127)
    assert (flags & 4) == 0
    err = np.abs(y.astype(np.int64) - want)
    assert err.max() > 0                          # gaussian sigma-32 filters do get scaled
    assert err.mean() < 0.02 * np.abs(want).mean()


# ---- the paper's own setting: uint8 values minus their zero point (int9), Section 4.1 ---------------------------

def test_int16_direct_convolution_against_int8_and_einsum():
    x, g = wl.make_custom(2, 3, 4, 5, 6, seed=10)
    assert np.array_equal(oracle.direct_conv2d_i16(x.astype(np.int16), g.astype(np.int16)), oracle.direct_conv2d(x, g))
    rng = np.random.default_rng(11)
    x9 = rng.integers(-255, 256, (2, 3, 5, 6)).astype(np.int16)
    g9 = rng.integers(-255, 256, (4, 3, 3, 3)).astype(np.int16)
    xp = np.pad(x9.astype(np.int64), ((0, 0), (0, 0), (1, 1), (1, 1)))
    want = sum(np.einsum("nchw,kc->nkhw", xp[:, :, a:a + 5, b:b + 6], g9[:, :, a, b].astype(np.int64))
               for a in range(3) for b in range(3))
    assert np.array_equal(oracle.direct_conv2d_i16(x9, g9), want.astype(np.int32))


def test_int9_filters_reach_the_printed_worst_case_entries():
    """All taps at +255 (uint8 255, zero point 0) give 4, 6 and 9 times 255 at the corner, edge and centre entries:
    the 1020 / 1530 / 2295 of the printed table, which need 11 / 12 / 13 bits."""
    gold = golden_io.sections("f2x2_3x3_worstcase.txt")
    Wt = oracle.f2_filter_transform_i16(np.full((1, 1, 3, 3), 255, np.int16))[0, 0]
    mag = np.real(gold["MAG"]).astype(np.int64)
    for (r, c) in ((0, 0), (0, 1), (1, 0), (1, 1), (3, 3), (0, 3), (3, 1)):
        assert Wt[r, c] == mag[r, c]
    assert np.all(np.abs(Wt) <= mag)
    corners = np.array(list(itertools.product([-255, 255], repeat=9)), np.int16).reshape(-1, 1, 3, 3)
    assert np.array_equal(np.abs(oracle.f2_filter_transform_i16(corners)).max(axis=(0, 1)), mag)


def test_int9_lossless_equals_direct_and_scaling_to_the_papers_range():
    rng = np.random.default_rng(12)
    x9 = (rng.integers(0, 256, (2, 5, 7, 6)) - 117).astype(np.int16)        # uint8 activations, zero point 117
    g9 = (rng.integers(0, 256, (3, 5, 3, 3)) - 131).astype(np.int16)        # uint8 weights, zero point 131
    want = oracle.direct_conv2d_i16(x9, g9)
    y, flags = oracle.f2_conv2d_i16(x9, g9, oracle.LOSSLESS)
    assert flags == 0 and np.array_equal(y, want)
    for rng_ in (127, 255):                                                 # int8 operands / the paper's int9
        scaled, tab, mx = oracle.f2_scale_filters(oracle.f2_filter_transform_i16(g9), rng_)
        assert np.abs(scaled).max() <= rng_ and (tab[..., 0] != 0).any()
        y, flags = oracle.f2_conv2d_i16(x9, g9, oracle.SCALED, rng_)
        err = np.abs(y.astype(np.int64) - want)
        assert (flags & 4) == 0 and err.mean() < 0.02 * np.abs(want).mean()


# ---- activations scaled as well (the remark that closes Section 4.1; rule of Section 4.2 per tile) ---------------

def test_activation_scaling_follows_the_rule_per_tile_and_location():
    x, _ = wl.make_custom(2, 10, 1, 7, 6, seed=13)
    D = oracle.f2_input_transform(x)
    assert np.abs(D).max() <= 4 * 128                     # the 11 bits Section 4.1 states for int8 data
    scaled, tab, mx = oracle.f2_scale_activations(D, 127)
    assert np.array_equal(mx, np.abs(D).max(axis=1)) and np.abs(scaled).max() <= 127
    for t in range(D.shape[0]):
        for r in range(4):
            for c in range(4):
                n, p = oracle.scale_factor(int(mx[t, r, c]), 127)
                rr, q = oracle.inverse_factor(n, p)
                assert tuple(tab[t, r, c]) == (n, p, rr, q)
                want = D[t, :, r, c] if n == 0 else (D[t, :, r, c] * n + (1 << (p - 1))) >> p
                assert np.array_equal(scaled[t, :, r, c], want)
    assert (tab[..., 0] != 0).any() and (tab[..., 0] == 0).any()
    # a tile's operands depend on that tile alone
    one, tab1, _ = oracle.f2_scale_activations(D[5:6], 127)
    assert np.array_equal(one[0], scaled[5]) and np.array_equal(tab1[0], tab[5])


def test_both_scaled_equals_filter_scaled_when_no_tile_needs_scaling():
    """|x| <= 31 keeps |B^T d B| <= 4 * 31 within the range, so no activation factor is applied."""
    rng = np.random.default_rng(14)
    x = rng.integers(-31, 32, (2, 9, 6, 7)).astype(np.int8)
    _, g = wl.make_custom(1, 9, 5, 6, 7, seed=15)
    assert np.abs(oracle.f2_input_transform(x)).max() <= 127
    y1, _ = oracle.f2_conv2d(x, g, oracle.SCALED, 127)
    y2, flags = oracle.f2_conv2d(x, g, oracle.BOTH_SCALED, 127)
    assert (flags & 4) == 0 and np.array_equal(y1, y2)
    assert not np.array_equal(y1, oracle.direct_conv2d(x, g))       # the filters were scaled
    # with a range nothing exceeds, both reduce to the direct convolution
    x, g = wl.make_custom(1, 6, 3, 6, 6, seed=16)
    y, _ = oracle.f2_conv2d(x, g, oracle.BOTH_SCALED, 1 << 20)
    assert np.array_equal(y, oracle.direct_conv2d(x, g))


def test_both_scaled_reverses_the_activation_factor_after_the_filter_factor():
    """One channel, one tile: the result can be followed by hand from the two tables."""
    x = np.zeros((1, 1, 2, 2), np.int8)
    x[0, 0] = [[127, -128], [90, 127]]
    g = np.full((1, 1, 3, 3), 100, np.int8)
    D = oracle.f2_input_transform(x)
    Wt = oracle.f2_filter_transform(g)
    Ds, ta, _ = oracle.f2_scale_activations(D, 127)
    Ws, tf, _ = oracle.f2_scale_filters(Wt, 127)
    assert (ta[..., 0] != 0).any() and (tf[..., 0] != 0).any()
    M = np.zeros((4, 4), np.int64)
    for r in range(4):
        for c in range(4):
            s = int(Ws[0, 0, r, c] * Ds[0, 0, r, c])
            for n, p, rr, q in (tf[0, r, c], ta[0, r, c]):
                if n != 0:
                    s = (s * int(rr) + (1 << (int(q) - 1) if q else 0)) >> int(q)
            M[r, c] = s
    _, _, at = oracle.f2_matrices()
    want = ((at @ M @ at.T) + 2) >> 2
    y, _ = oracle.f2_conv2d(x, g, oracle.BOTH_SCALED, 127)
    assert np.array_equal(y[0, 0], want)


def test_both_scaled_error_is_small_relative_to_signal():
    x, g = wl.make_custom(2, 32, 8, 12, 12, act="relu", wgt="gauss", seed=9)
    want = oracle.direct_conv2d(x, g).astype(np.int64)
    y1, _ = oracle.f2_conv2d(x, g, oracle.SCALED, 127)
    y2, flags = oracle.f2_conv2d(x, g, oracle.BOTH_SCALED, 127)
    assert (flags & 4) == 0 and not np.array_equal(y1, y2)          # post-ReLU activations do get scaled
    assert np.abs(y2.astype(np.int64) - want).mean() < 0.03 * np.abs(want).mean()
