"""Pins for the oracle's activation-side scaling on the complex F(4x4,3x3) path (the remark that closes Section 4.1,
read as Section 4.2's rule with a tile in the place of an output feature map).  No GPU."""
import numpy as np

import oracle
from paper_1901_01965_amd import workloads as wl


def test_activation_scaling_follows_the_rule_per_tile_and_location():
    x, _ = wl.make_custom(2, 10, 1, 9, 7, act="uniform", seed=13)
    D = oracle.input_transform(x)
    assert np.abs(D).max() <= 16 * 128                    # 12 bits for int8 data (Section 3.4)
    scaled, tab, mx = oracle.scale_activations(D, 127)
    assert np.array_equal(mx, np.abs(D).max(axis=(1, 4))) and np.abs(scaled).max() <= 127
    pm = oracle.partner_map()
    for t in range(D.shape[0]):
        for r in range(6):
            for c in range(6):
                n, p = oracle.scale_factor(int(mx[t, r, c]), 127)
                rr, q = oracle.inverse_factor(n, p)
                assert tuple(tab[t, r, c]) == (n, p, rr, q)
                want = D[t, :, r, c] if n == 0 else (D[t, :, r, c] * n + (1 << (p - 1))) >> p
                pr, pc = pm[r, c]
                if (pr, pc) == (r, c):
                    # a canonical location: Re and Im each multiplied and rounded half up
                    assert np.array_equal(scaled[t, :, r, c], want)
                else:
                    # the conjugate of its canonical partner's scaled value (and the partner's table entry)
                    assert np.array_equal(scaled[t, :, r, c], scaled[t, :, pr, pc] * np.array([1, -1]))
                    assert np.array_equal(tab[t, r, c], tab[t, pr, pc])
    # the 26 canonical locations: 16 stay real, 10 are complex
    canonical = [(r, c) for r in range(6) for c in range(6) if tuple(pm[r, c]) == (r, c)]
    assert len(canonical) == 26 and sum(1 for (r, c) in canonical if np.any(D[:, :, r, c, 1])) == 10
    assert (tab[..., 0] != 0).any() and (tab[..., 0] == 0).any()
    # a tile's operands depend on that tile alone
    one, tab1, _ = oracle.scale_activations(D[5:6], 127)
    assert np.array_equal(one[0], scaled[5]) and np.array_equal(tab1[0], tab[5])


def test_both_scaled_equals_filter_scaled_when_no_tile_needs_scaling():
    """|x| <= 7 keeps |B^T d B| <= 16 * 7 within the range, so no activation factor is applied."""
    rng = np.random.default_rng(14)
    x = rng.integers(-7, 8, (2, 9, 6, 7)).astype(np.int8)
    _, g = wl.make_custom(1, 9, 5, 6, 7, seed=15)
    assert np.abs(oracle.input_transform(x)).max() <= 127
    y1, _ = oracle.winograd_conv2d(x, g, oracle.SCALED, 127)
    y2, flags = oracle.winograd_conv2d(x, g, oracle.BOTH_SCALED, 127)
    assert (flags & 5) == 0 and np.array_equal(y1, y2)
    assert not np.array_equal(y1, oracle.direct_conv2d(x, g))       # the filters were scaled
    # with a range nothing exceeds, both reduce to the direct convolution
    x, g = wl.make_custom(1, 6, 3, 6, 6, seed=16)
    y, _ = oracle.winograd_conv2d(x, g, oracle.BOTH_SCALED, 1 << 20)
    assert np.array_equal(y, oracle.direct_conv2d(x, g))


def test_both_scaled_pipeline_followed_by_hand_on_one_tile():
    """One tile, one channel, one filter; every number below worked out by hand (none comes from the oracle).

    Filter as in the filter-scaled by-hand case: taps g[0][0] = 81, g[0][1] = 56, so G' g G'^T has row 0 =
    (1296, 548, 100, 324+224i, 324-224i, 0), factors (12,7,171,4), (14,6,146,5), none, (12,5,171,6), scaled row
    (122, 120, 100, 122+84i, 122-84i, 0).
    Image 8x8 with x[3][3..7] = (120, 100, 90, -60, 50): tile (1,1) reads rows and columns 3..8, so only the first row
    of its patch is non-zero, v = (120, 100, 90, -60, 50, 0), and B^T d B has row 0 =
      (v0-v4, v1+v2+v3+v4, -v1+v2-v3+v4, (v4-v2) + i(v3-v1), conjugate, v5-v1) = (70, 180, 100, -40-160i, -40+160i, -100).
    Tile factors (range 127; x = 127*128/max, y = floor(log2 x), n = floor(x/2^(y-3)), p = 10-y):
      180: x = 90.3, y = 6, n = 11, p = 4; reciprocal 2^(4+q)/11 <= 255 -> q = 7, r = round(186.2) = 186
      160 (the larger of |Re|, |Im|): x = 101.6, y = 6, n = 12, p = 4; 2^(4+q)/12 -> q = 7, r = round(170.7) = 171
      70, 100, 100: within the range.
    Scaled activations, round half up: (180*11 + 8) >> 4 = 124; (-40*12 + 8) >> 4 = floor(-29.5) = -30;
      (-160*12 + 8) >> 4 = floor(-119.5) = -120.
    Products: 122*70 = 8540; 120*124 = 14880; 100*100 = 10000; (122+84i)(-30-120i) = 6420 - 17160i; 0.
    Filter's reciprocal first: (8540*171 + 8) >> 4 = 91271; (14880*146 + 16) >> 5 = 67890; 10000;
      (6420*171 + 32) >> 6 = 17153; (-17160*171 + 32) >> 6 = floor(-45848.9) = -45849.
    Then the tile's: 91271; (67890*186 + 64) >> 7 = 98653; 10000; (17153*171 + 64) >> 7 = 22915;
      (-45849*171 + 64) >> 7 = floor(-61250.9) = -61251.
      (The other order would give (14880*186 + 64) >> 7 = 21623, then (21623*146 + 16) >> 5 = 98655 at entry (0,1).)
    Output row 0, m3 = 22915 - 61251i:
      Y0 = 91271 + 98653 + 10000 + 2*22915 = 245754      Y1 = 98653 - 10000 + 2*61251 = 211155
      Y2 = 98653 + 10000 - 2*22915 = 62823               Y3 = 98653 - 10000 - 2*61251 + 0 = -33849
    y = (Y + 8) >> 4 = (15360, 13197, 3926, -2116); the exact convolution there is (15320, 13140, 3930, -2060)."""
    x = np.zeros((1, 1, 8, 8), np.int8)
    x[0, 0, 3, 3:8] = [120, 100, 90, -60, 50]
    g = np.zeros((1, 1, 3, 3), np.int8)
    g[0, 0, 0, 0], g[0, 0, 0, 1] = 81, 56
    t = 3
    assert list(oracle.direct_conv2d(x, g)[0, 0, 4, 4:8]) == [15320, 13140, 3930, -2060]

    D = oracle.input_transform(x)
    assert np.array_equal(D[t, 0, 0], [[70, 0], [180, 0], [100, 0], [-40, -160], [-40, 160], [-100, 0]])
    assert not D[t, 0, 1:].any()
    Ds, atab, amx = oracle.scale_activations(D, 127)
    assert [tuple(atab[t, 0, c]) for c in range(6)] == [(0, 0, 1, 0), (11, 4, 186, 7), (0, 0, 1, 0), (12, 4, 171, 7),
                                                         (12, 4, 171, 7), (0, 0, 1, 0)]
    assert list(amx[t, 0]) == [70, 180, 100, 160, 160, 100]
    assert np.array_equal(Ds[t, 0, 0], [[70, 0], [124, 0], [100, 0], [-30, -120], [-30, 120], [-100, 0]])

    Ws, tab, _ = oracle.scale_filters(oracle.filter_transform(g), 127)
    assert np.array_equal(Ws[0, 0, 0], [[122, 0], [120, 0], [100, 0], [122, 84], [122, -84], [0, 0]])
    Mt = oracle.contract(Ds, Ws)
    assert np.array_equal(Mt[t, 0, 0], [[8540, 0], [14880, 0], [10000, 0], [6420, -17160], [6420, 17160], [0, 0]])
    Mf = oracle.inverse_scale(Mt, tab)
    assert np.array_equal(Mf[t, 0, 0], [[91271, 0], [67890, 0], [10000, 0], [17153, -45849], [17153, 45849], [0, 0]])
    M = oracle.inverse_scale_tiles(Mf, atab)
    assert np.array_equal(M[t, 0, 0], [[91271, 0], [98653, 0], [10000, 0], [22915, -61251], [22915, 61251], [0, 0]])
    assert not M[t, 0, 1:].any()
    # the order matters at entry (0,1)
    other = oracle.inverse_scale(oracle.inverse_scale_tiles(Mt, atab), tab)
    assert other[t, 0, 0, 1, 0] == 98655 != M[t, 0, 0, 1, 0]

    y16, flags = oracle.output_transform(M, 1, 1, 8, 8, shift=0)
    assert flags == 0 and list(y16[0, 0, 4, 4:8]) == [245754, 211155, 62823, -33849]
    yy, flags = oracle.winograd_conv2d(x, g, oracle.BOTH_SCALED, 127)
    assert (flags & 5) == 0
    assert list(yy[0, 0, 4, 4:8]) == [15360, 13197, 3926, -2116] and not yy[0, 0, 5:8, 4:8].any()


def test_both_scaled_error_is_small_relative_to_signal():
    x, g = wl.make_custom(2, 32, 8, 12, 12, act="relu", wgt="gauss", seed=9)
    want = oracle.direct_conv2d(x, g).astype(np.int64)
    y1, _ = oracle.winograd_conv2d(x, g, oracle.SCALED, 127)
    y2, flags = oracle.winograd_conv2d(x, g, oracle.BOTH_SCALED, 127)
    assert (flags & 5) == 0 and not np.array_equal(y1, y2)          # post-ReLU activations do get scaled
    assert np.abs(y2.astype(np.int64) - want).mean() < 0.03 * np.abs(want).mean()
