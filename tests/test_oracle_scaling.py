"""Pins for the CPU oracle's bit-width analysis and filter precision scaling
(Sections 4.1-4.3 of the paper).  No GPU.

The general lossy result of the scaled path has no printed worked example:
it is PARITY UNPINNED beyond the special cases and statistics checked here.
"""
import itertools
import math

import numpy as np
import pytest

import oracle
from tests import golden_io
from paper_1901_01965_amd import workloads as wl

CONST = golden_io.constants()


def _cx(a):
    return a[..., 0] + 1j * a[..., 1]


# ----------------------------------------------------------------------------
# Section 4.1: worst-case magnitudes and bit widths

def _bits_signed(mag):
    """Bits of a two's-complement field that holds every value in [-mag, mag]."""
    return int(mag).bit_length() + 1


def test_f2x2_worstcase_table_is_the_printed_one():
    gold = golden_io.sections("f2x2_3x3_worstcase.txt")
    re, im = oracle.worstcase_magnitude(gold["GP"], 255, 255)
    assert np.array_equal(re, np.real(gold["MAG"]).astype(np.int64))
    assert not im.any()
    bits = np.vectorize(_bits_signed)(re)
    assert np.array_equal(bits, np.real(gold["BITS"]).astype(np.int64))
    assert re.max() == CONST["f2x2_max_magnitude"]
    assert bits.max() == CONST["scaled_filter_bits_before"]


def test_worstcase_routine_against_vertex_enumeration():
    """Every entry of G' g G'^T is linear in the 9 taps, so its extremes over a box sit
    at the box's 512 corners: enumerate them."""
    _, g4, _ = oracle.matrices()
    corners = np.array(list(itertools.product([-128, 127], repeat=9)), np.float64).reshape(-1, 3, 3)
    Wt = np.einsum("ra,nab,sb->nrs", g4, corners, g4)
    re, im = oracle.worstcase_magnitude(g4, 127, 128)
    assert np.array_equal(re, np.abs(np.real(Wt)).max(0).astype(np.int64))
    assert np.array_equal(im, np.abs(np.imag(Wt)).max(0).astype(np.int64))


def test_complex_filter_transform_widens_int8_by_four_bits():
    """Section 3.4: 8 + ceil(log2(4^2)) = 12 bits hold every transformed int8 filter entry."""
    _, g4, _ = oracle.matrices()
    corners = np.array(list(itertools.product([-128, 127], repeat=9)), np.float64).reshape(-1, 3, 3)
    Wt = np.einsum("ra,nab,sb->nrs", g4, corners, g4)
    bits = 8 + int(CONST["filter_widening_bits_complex"])
    lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    for part in (np.real(Wt), np.imag(Wt), np.real(Wt) + np.imag(Wt)):   # the sum feeds the 3-mult product
        assert part.min() >= lo and part.max() <= hi
    assert np.real(Wt).min() == lo                                        # the bound is tight
    assert math.ceil(math.log2(24 ** 2)) == CONST["filter_widening_bits_rational"]
    assert round(100 * (1 - (8 + 4) / (8 + 10)), 2) == CONST["bitwidth_reduction_vs_rational"]
    assert round(100 * ((3.13 / 12) / (4.0 / 18) - 1), 2) == CONST["efficiency_gain_vs_rational_f4"]
    assert round(100 * ((3.13 / 12) / (2.25 / 10) - 1), 2) == CONST["efficiency_gain_vs_rational_f2"]


def test_rational_f4x4_needs_eighteen_bits_where_the_complex_algorithm_needs_twelve():
    """Section 3.2: the rational F(4x4,3x3) matrix G (points 0, +-1, +-2) has the denominator 24, so exact integer
    arithmetic needs G' = 24 G and widens an int8 filter by ceil(log2(24^2)) = 10 bits.  The oracle's worst-case routine
    (pinned to the printed 1020/1530/2295 table) on that G' and on the complex G' = 4 G gives the two bit widths the
    33.33 % of Section 3.4 compares."""
    g_rat = np.real(golden_io.sections("rational_f4x4_3x3_filter_matrix.txt")["G"])
    g24 = np.rint(24 * g_rat)
    assert np.allclose(24 * g_rat, g24) and not np.allclose(12 * g_rat, np.rint(12 * g_rat))   # 24 is the least multiplier
    re, im = oracle.worstcase_magnitude(g24.astype(np.complex128), 127, 128)
    assert not im.any()
    assert re.max() == 24 * 24 * 128 and re[5, 5] == re.max()         # the corner entry passes a tap through (24 * 1)^2
    bits_rational = int(re.max()).bit_length() + 1                     # signed
    corners = np.array(list(itertools.product([-128, 127], repeat=9)), np.float64).reshape(-1, 3, 3)
    assert np.abs(np.einsum("ra,nab,sb->nrs", g24, corners, g24)).max() == re.max()   # reached by a box corner
    _, g4, _ = oracle.matrices()
    re_c, im_c = oracle.worstcase_magnitude(g4, 127, 128)
    bits_complex = int(max(re_c.max(), im_c.max()) - 1).bit_length() + 1   # -2048 itself still fits 12 bits
    assert (bits_rational, bits_complex) == (8 + int(CONST["filter_widening_bits_rational"]),
                                             8 + int(CONST["filter_widening_bits_complex"])) == (18, 12)
    assert round(100 * (1 - bits_complex / bits_rational), 2) == CONST["bitwidth_reduction_vs_rational"]


def test_transformed_activations_fit_twelve_bits():
    """B^T d B of int8 data, and the real+imaginary sum the 3-mult product needs, fit 12 bits."""
    re, im = oracle.worstcase_input_magnitude(127, 128)
    assert re.max() <= 2048 and im.max() <= 1024
    # brute force on sign patterns that maximise each entry
    bt, _, _ = oracle.matrices()
    coef = np.einsum("ra,sb->rsab", bt, bt)                  # D[r,s] = sum coef[r,s,a,b] d[a,b]
    for part, bound in ((np.real(coef), re), (np.imag(coef), im)):
        hi = np.where(part > 0, 127, -128) * part
        lo = np.where(part > 0, -128, 127) * part
        assert np.array_equal(np.maximum(hi.sum((2, 3)), -lo.sum((2, 3))).astype(np.int64), bound)
        assert hi.sum((2, 3)).max() <= 2047 and lo.sum((2, 3)).min() >= -2048
    both = np.real(coef) + np.imag(coef)
    hi = (np.where(both > 0, 127, -128) * both).sum((2, 3))
    lo = (np.where(both > 0, -128, 127) * both).sum((2, 3))
    assert hi.max() <= 2047 and lo.min() >= -2048


# ----------------------------------------------------------------------------
# Section 4.2: the down-scale factor n / 2^p

def _best_factor_brute_force(mx, rng_):
    """Largest n / 2^p with n in 1..15 and p in 4..8 that keeps n*mx <= range*2^p."""
    best = None
    for p in range(4, 9):
        for n in range(1, 16):
            if n * mx <= rng_ * (1 << p):
                f = n / (1 << p)
                if best is None or f > best:
                    best = f
    return best


def test_scale_factor_for_the_papers_int9_example():
    t1 = golden_io.table1()
    seen_p = set()
    for mx in range(1, 2296):
        n, p = oracle.scale_factor(mx, 255)
        if mx <= 255:
            assert (n, p) == (0, 0)                          # "no scaling", code 0
            continue
        assert 8 <= n <= 15                                  # normalised 4-bit n
        assert CONST["scale_p_min"] <= p <= CONST["scale_p_max"]
        seen_p.add(p)
        val, grey = t1[(n, p - 4)]
        assert not grey                                      # only non-grey entries of Table 1 are used
        assert abs(val - n / (1 << p)) < 6e-6
        assert n * mx <= 255 * (1 << p)                      # back inside the int9 range
        assert n / (1 << p) == _best_factor_brute_force(mx, 255)
    assert seen_p == {4, 5, 6, 7}
    assert oracle.scale_factor(2295, 255) == (14, 7)         # 1/9 rounded down: 0.10938
    assert oracle.scale_factor(256, 255) == (15, 4)          # 0.93750


def test_table1_is_n_over_two_to_p_plus_4():
    for (n, P), (val, _) in golden_io.table1().items():
        assert abs(val - n / (1 << (P + 4))) < 6e-6


def test_scale_factor_for_int8_filters():
    """Signed int8 weights: range 127; transformed magnitudes reach 16*128 = 2048."""
    for mx in range(1, 2049):
        n, p = oracle.scale_factor(mx, 127)
        if mx <= 127:
            assert (n, p) == (0, 0)
            continue
        assert 8 <= n <= 15 and 4 <= p <= 8
        if mx <= 2032:                                       # |g| <= 127 gives at most 16*127
            assert p <= 7
        assert n * mx <= 127 * (1 << p)
        assert n / (1 << p) == _best_factor_brute_force(mx, 127)


def test_scaled_filters_return_to_nine_bits():
    """Section 4.3: 13-bit Winograd-domain filters come back to 9 bits: 30.77% fewer."""
    for mx in range(256, 2296):
        n, p = oracle.scale_factor(mx, 255)
        for v in (mx, -mx):
            s = oracle.scale_round(v, n, p)
            assert -255 <= s <= 255
    before, after = CONST["scaled_filter_bits_before"], CONST["scaled_filter_bits_after"]
    assert _bits_signed(255) == after
    assert round(100 * (1 - after / before), 2) == CONST["scaled_filter_bits_reduction"]


def test_inverse_factor_is_eight_bit_multiply_and_shift():
    shifts = set()
    for mx in range(256, 2296):
        n, p = oracle.scale_factor(mx, 255)
        r, q = oracle.inverse_factor(n, p)
        assert 1 <= r < (1 << int(CONST["inverse_multiplier_bits"]))
        assert CONST["inverse_shift_min"] <= q <= CONST["inverse_shift_max"]
        shifts.add(q)
        exact = (1 << p) / n
        assert abs(r / (1 << q) - exact) <= 0.5 / (1 << q)   # nearest multiple of 2^-q
        if q < 7:                                            # one more bit would overflow 8 bits
            assert round(exact * (1 << (q + 1))) > 255
    assert shifts == {4, 5, 6, 7}
    assert oracle.inverse_factor(0, 0) == (1, 0)
    assert oracle.inverse_factor(15, 8) == (137, 3)          # int8 extension: 2^8/15 = 17.07
    assert oracle.inverse_factor(8, 7) == (128, 3)           # reciprocal 16 needs shift 3


def test_rounding_is_half_up():
    assert oracle.scale_round(5, 1, 1) == 3
    assert oracle.scale_round(-5, 1, 1) == -2
    assert oracle.scale_round(7, 3, 2) == 5                  # 21/4 = 5.25
    assert oracle.scale_round(-7, 3, 2) == -5
    assert oracle.scale_round(9, 7, 0) == 63


def test_down_then_up_error_statistics():
    """Section 4.3 reports a small positive-biased static error: mean 1.12, about 0.1%.
    Modelled over every scalable int9 magnitude; a weak pin on the rounding choices
    (truncation in either direction gives a clearly negative mean)."""
    err, rel = [], []
    for mx in range(256, 2296):
        n, p = oracle.scale_factor(mx, 255)
        r, q = oracle.inverse_factor(n, p)
        back = oracle.scale_round(oracle.scale_round(mx, n, p), r, q)
        err.append(back - mx)
        rel.append((back - mx) / mx)
    assert 0.5 < np.mean(err) < 2.0
    assert 0.0005 < np.mean(rel) < 0.002


# ----------------------------------------------------------------------------
# the scaled filters and the scaled pipeline

def test_scale_filters_structure():
    _, g = wl.make_custom(1, 6, 5, 4, 4, wgt="gauss", seed=21)
    Wt = oracle.filter_transform(g)
    Ws, tab, mx = oracle.scale_filters(Wt, 127)
    pm = oracle.partner_map()
    assert np.abs(Ws).max() <= 127                           # back in the spatial weight range
    for r in range(6):
        for c in range(6):
            pr, pc = pm[r, c]
            canonical = (pr, pc) == (r, c)
            want_mx = np.abs(Wt[:, :, r, c, :]).max(axis=(1, 2))
            assert np.array_equal(mx[:, r, c], want_mx)
            for k in range(g.shape[0]):
                n, p, rr, q = tab[k, r, c]
                assert (n, p) == oracle.scale_factor(int(want_mx[k]), 127)
                assert (rr, q) == oracle.inverse_factor(n, p)
                if canonical:
                    if n == 0:
                        assert np.array_equal(Ws[k, :, r, c], Wt[k, :, r, c])
                    else:
                        want = (Wt[k, :, r, c] * n + (1 << (p - 1))) >> p
                        assert np.array_equal(Ws[k, :, r, c], want)
                else:                                        # partners are conjugates of the scaled entry
                    assert np.array_equal(Ws[k, :, r, c, 0], Ws[k, :, pr, pc, 0])
                    assert np.array_equal(Ws[k, :, r, c, 1], -Ws[k, :, pr, pc, 1])


def test_scaled_equals_direct_when_no_location_needs_scaling():
    """|g| <= 7 keeps every transformed magnitude <= 16*7 = 112 <= 127."""
    x, _ = wl.make_custom(1, 4, 3, 9, 6, seed=22)
    g = np.random.default_rng(22).integers(-7, 8, (3, 4, 3, 3)).astype(np.int8)
    y, flags = oracle.winograd_conv2d(x, g, oracle.SCALED, 127)
    assert flags == 0
    assert np.array_equal(y, oracle.direct_conv2d(x, g))


def test_scaled_with_huge_range_equals_lossless():
    x, g = wl.make_custom(2, 3, 3, 6, 7, seed=23)
    y, flags = oracle.winograd_conv2d(x, g, oracle.SCALED, 1 << 20)
    assert flags == 0
    assert np.array_equal(y, oracle.direct_conv2d(x, g))


def test_unscaled_locations_contribute_exactly():
    """Locations whose maximum is within range are identical in both modes (stage level)."""
    x, g = wl.make_custom(1, 4, 2, 8, 8, wgt="gauss", seed=24)
    D = oracle.input_transform(x)
    Wt = oracle.filter_transform(g)
    Ws, tab, _ = oracle.scale_filters(Wt, 127)
    M = oracle.contract(D, Wt)
    Ms = oracle.inverse_scale(oracle.contract(D, Ws), tab)
    unscaled = tab[..., 0] == 0                              # [K,6,6]
    for k in range(2):
        assert np.array_equal(Ms[:, k][:, unscaled[k]], M[:, k][:, unscaled[k]])
    # and the scaled ones stay conjugate-symmetric, so the output is real
    y, flags = oracle.output_transform(Ms, 1, 2, 8, 8, shift=4, round_add=8)
    assert (flags & 1) == 0


def test_scaled_error_is_small_relative_to_signal():
    x, g = wl.make_custom(2, 16, 8, 12, 12, act="relu", wgt="gauss", seed=25)
    y, flags = oracle.winograd_conv2d(x, g, oracle.SCALED, 127)
    assert (flags & 5) == 0
    d = oracle.direct_conv2d(x, g).astype(np.int64)
    err = np.abs(y.astype(np.int64) - d)
    assert err.mean() < 0.02 * np.abs(d).mean()
    assert err.max() > 0                                      # it is a lossy mode


def test_scaled_f4x4_pipeline_followed_by_hand_on_one_tile():
    """One tile, one channel, one filter, every number below worked out by hand from Section 4.2's steps
    (none of them comes from the oracle).

    Filter taps g[0][0] = 81, g[0][1] = 56: with a = (4,1,1,1,1,0) and b = (0,1,-1,i,-i,0), the first two
    columns of G' = 4G, G' g G'^T has row 0 = 4 (81 a + 56 b) = (1296, 548, 100, 324+224i, 324-224i, 0).
    Image 8x8 with x[3][3] = 88, x[3][4] = -38: tile (1,1) reads rows and columns 3..8, so its patch is
    88, -38 in the first row, and B^T d B has row 0 = (88, -38, 38, 38i, -38i, 38), every other row zero.

    Scale factors (range 127): x = 127*128/max, y = floor(log2 x), n = floor(x / 2^(y-3)), p = 10 - y:
      1296: x = 12.54, y = 3, n = 12, p = 7;  reciprocal 2^(7+q)/12 <= 255 -> q = 4, r = round(170.67) = 171
       548: x = 29.66, y = 4, n = 14, p = 6;  2^(6+q)/14 -> q = 5, r = round(146.29) = 146
       100: within the range, not scaled
       324: x = 50.17, y = 5, n = 12, p = 5;  2^(5+q)/12 -> q = 6, r = 171   (Re and Im share it)
    Scaled filters, round half up: (1296*12 + 64) >> 7 = 122, (548*14 + 32) >> 6 = 120,
      (324*12 + 16) >> 5 = 122, (224*12 + 16) >> 5 = 84.
    Products (one channel): 122*88 = 10736; 120*(-38) = -4560; 100*38 = 3800; (122+84i)(38i) = -3192 + 4636i.
    Scaled back: (10736*171 + 8) >> 4 = 114741; (-4560*146 + 16) >> 5 = floor(-20804.5) = -20805; 3800;
      (-3192*171 + 32) >> 6 = floor(-8528.1) = -8529; (4636*171 + 32) >> 6 = 12387.
    Output transform: only row 0 of M is non-zero and A^T has a single 1 in its first column, so only output
    row 0 is non-zero: with m3 = -8529 + 12387i,
      Y0 = 114741 - 20805 + 3800 + 2(-8529) = 80678     Y1 = -20805 - 3800 - 2(12387) = -49379
      Y2 = -20805 + 3800 - 2(-8529) = 53                Y3 = -20805 - 3800 + 2(12387) + 0 = 169
    and y = (Y + 8) >> 4 = (5042, -3086, 3, 11); the exact convolution there is (5000, -3078, 0, 0).
    80678 = 16*5042 + 6: shifting by 2 with rounding after each 1-D transform instead (which equals
    floor((Y + 10) / 16)) would give 5043, so this case tells the two conventions apart."""
    x = np.zeros((1, 1, 8, 8), np.int8)
    x[0, 0, 3, 3], x[0, 0, 3, 4] = 88, -38
    g = np.zeros((1, 1, 3, 3), np.int8)
    g[0, 0, 0, 0], g[0, 0, 0, 1] = 81, 56
    t = 3   # tile (ty, tx) = (1, 1) of the 2x2 tiles

    D = oracle.input_transform(x)
    want_row0 = np.array([[88, 0], [-38, 0], [38, 0], [0, 38], [0, -38], [38, 0]])
    assert np.array_equal(D[t, 0, 0], want_row0) and not D[t, 0, 1:].any()

    Wt = oracle.filter_transform(g)
    assert np.array_equal(Wt[0, 0, 0], [[1296, 0], [548, 0], [100, 0], [324, 224], [324, -224], [0, 0]])
    Ws, tab, mx = oracle.scale_filters(Wt, 127)
    assert [tuple(tab[0, 0, c]) for c in range(5)] == [(12, 7, 171, 4), (14, 6, 146, 5), (0, 0, 1, 0),
                                                        (12, 5, 171, 6), (12, 5, 171, 6)]
    assert list(mx[0, 0]) == [1296, 548, 100, 324, 324, 0]
    assert np.array_equal(Ws[0, 0, 0], [[122, 0], [120, 0], [100, 0], [122, 84], [122, -84], [0, 0]])

    Mt = oracle.contract(D, Ws)
    assert np.array_equal(Mt[t, 0, 0], [[10736, 0], [-4560, 0], [3800, 0], [-3192, 4636], [-3192, -4636], [0, 0]])
    M = oracle.inverse_scale(Mt, tab)
    assert np.array_equal(M[t, 0, 0], [[114741, 0], [-20805, 0], [3800, 0], [-8529, 12387], [-8529, -12387], [0, 0]])
    assert not M[t, 0, 1:].any()

    y16, flags = oracle.output_transform(M, 1, 1, 8, 8, shift=0)
    assert flags == 0 and list(y16[0, 0, 4, 4:8]) == [80678, -49379, 53, 169]
    y, flags = oracle.output_transform(M, 1, 1, 8, 8, shift=4, round_add=8)
    assert flags == 0
    assert list(y[0, 0, 4, 4:8]) == [5042, -3086, 3, 11] and not y[0, 0, 5:8, 4:8].any()

    # the whole pipeline in one call gives the same tile, and is not the per-stage-shift variant
    yy, flags = oracle.winograd_conv2d(x, g, oracle.SCALED, 127)
    assert (flags & 5) == 0
    assert list(yy[0, 0, 4, 4:8]) == [5042, -3086, 3, 11] and not yy[0, 0, 5:8, 4:8].any()
    assert (80678 + 10) // 16 == 5043 != yy[0, 0, 4, 4]
    assert list(oracle.direct_conv2d(x, g)[0, 0, 4, 4:8]) == [5000, -3078, 0, 0]
