"""GPU parity of the rational F(2x2,3x3) path, through the C ABI, bit for bit against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_1901_01965_amd as wg
from paper_1901_01965_amd import workloads as wl

pytestmark = pytest.mark.gpu

LAYOUTS = [wg.NHWC, wg.NCHW]
SHAPES = [  # N, C, K, H, W: ragged tiles, odd channel counts, several channel blocks, more than 32 tiles and filters
    (1, 1, 1, 1, 1), (1, 4, 4, 4, 4), (1, 3, 5, 7, 9), (2, 16, 16, 16, 16), (1, 70, 33, 10, 6), (3, 8, 100, 5, 13),
    (1, 130, 65, 8, 8), (2, 64, 64, 14, 14), (1, 200, 40, 6, 10),
]


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _x(x, layout):
    return _dev(x if layout == wg.NCHW else wl.to_nhwc(x))


def _g(g, layout):
    return _dev(g if layout == wg.NCHW else wl.to_krsc(g))


def _y(y, layout):
    y = y.cpu().numpy()
    return y if layout == wg.NCHW else wl.from_nhwc(y)


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("kc,wgt", [((4, 4), "uniform"), ((5, 3), "gauss"), ((64, 64), "gauss"), ((33, 70), "uniform")])
def test_filter_operands_and_scaling_table(kc, wgt, layout):
    """The blob's operand planes and (n, p, r, q) table against the oracle's G' g G'^T and Section 4.2 routine."""
    K, C = kc
    _, g = wl.make_custom(1, C, K, 4, 4, wgt=wgt, seed=70)
    Wt = oracle.f2_filter_transform(g)                      # [K, C, 4, 4]
    flat = Wt.reshape(K, C, 16).transpose(2, 0, 1)          # [16, K, C]
    planes, _ = wg.f2x2_debug_filter_operands(wg.f2x2_filter_transform(_g(g, layout), layout, wg.LOSSLESS))
    planes = planes.cpu().numpy().astype(np.int64)
    assert np.array_equal(planes[0::2], flat >> 6) and np.array_equal(planes[1::2], flat & 63)
    scaled, tab, _ = oracle.f2_scale_filters(Wt, 127)
    planes, table = wg.f2x2_debug_filter_operands(wg.f2x2_filter_transform(_g(g, layout), layout, wg.SCALED))
    assert np.array_equal(planes.cpu().numpy().astype(np.int64), scaled.reshape(K, C, 16).transpose(2, 0, 1))
    want = tab.reshape(K, 16, 4).copy()
    want[want[..., 0] == 0] = (0, 0, 1, 0)                  # the library stores "no scaling" as r/2^q = 1/1
    assert np.array_equal(table.cpu().numpy(), want)


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("shape", SHAPES)
def test_lossless_equals_oracle_direct(shape, layout):
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, seed=71)
    packed = wg.f2x2_filter_transform(_g(g, layout), layout, wg.LOSSLESS)
    y = wg.f2x2_conv2d_int8(_x(x, layout), packed, layout)
    assert np.array_equal(_y(y, layout), oracle.direct_conv2d(x, g))


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("wgt", ["uniform", "gauss"])
@pytest.mark.parametrize("shape", SHAPES)
def test_scaled_equals_oracle_scaled(shape, wgt, layout):
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, wgt=wgt, seed=72)
    want, flags = oracle.f2_conv2d(x, g, oracle.SCALED, 127)
    assert (flags & 4) == 0
    packed = wg.f2x2_filter_transform(_g(g, layout), layout, wg.SCALED)
    y = wg.f2x2_conv2d_int8(_x(x, layout), packed, layout)
    assert np.array_equal(_y(y, layout), want)


def test_extreme_values_and_many_channels():
    """All-extreme data at the largest supported channel count: every limb product and the joins at their limits."""
    C = wg.MAX_CHANNELS
    for xv, gv in ((-128, -128), (127, -128), (-128, 127)):
        x = np.full((1, C, 4, 6), xv, np.int8)
        g = np.full((2, C, 3, 3), gv, np.int8)
        g[1] = 127
        packed = wg.f2x2_filter_transform(_g(g, wg.NHWC), wg.NHWC, wg.LOSSLESS)
        y = wg.f2x2_conv2d_int8(_x(x, wg.NHWC), packed, wg.NHWC)
        assert np.array_equal(_y(y, wg.NHWC), oracle.direct_conv2d(x, g))


def test_cfg2_full_size_lossless_and_agreement_with_the_complex_algorithm():
    x, g = wl.make_case("cfg2")
    xd, gd = _x(x, wg.NHWC), _g(g, wg.NHWC)
    y2 = wg.f2x2_conv2d_int8(xd, wg.f2x2_filter_transform(gd, wg.NHWC, wg.LOSSLESS), wg.NHWC)
    y4 = wg.winograd_conv2d_int8(xd, wg.winograd_filter_transform(gd, wg.NHWC, wg.LOSSLESS), wg.NHWC)
    assert torch.equal(y2, y4)
    assert np.array_equal(_y(y2[:1], wg.NHWC), oracle.direct_conv2d(x[:1], g))


@pytest.mark.parametrize("name", ["cfg3", "cfg4a", "cfg4b"])
def test_full_size_scaled_configs(name):
    """The benchmark configurations at full size in the launch configuration bench.py --algorithm f2x2 times; the
    oracle checks the first and the last two images (tiles at both ends of the grid), the lossless result the whole
    batch against the direct kernel."""
    x, g = wl.make_case(name)
    xd, gd = _x(x, wg.NHWC), _g(g, wg.NHWC)
    y = _y(wg.f2x2_conv2d_int8(xd, wg.f2x2_filter_transform(gd, wg.NHWC, wg.SCALED), wg.NHWC), wg.NHWC)
    for sl in (slice(0, 1), slice(x.shape[0] - 2, x.shape[0])):
        want, flags = oracle.f2_conv2d(x[sl], g, oracle.SCALED, 127)
        assert (flags & 4) == 0
        assert np.array_equal(y[sl], want)
    lossless = wg.f2x2_conv2d_int8(xd, wg.f2x2_filter_transform(gd, wg.NHWC, wg.LOSSLESS), wg.NHWC)
    assert torch.equal(lossless, wg.direct_conv2d_int8(xd, gd, wg.NHWC))
    assert np.array_equal(_y(lossless[:1], wg.NHWC), oracle.direct_conv2d(x[:1], g))


def test_mismatched_blob_is_rejected_and_output_untouched():
    x, g = wl.make_custom(1, 8, 8, 6, 6, seed=73)
    packed = wg.f2x2_filter_transform(_g(g, wg.NHWC), wg.NHWC, wg.LOSSLESS)
    other = wg.F2x2PackedFilter(packed.blob, packed.K, packed.C, wg.SCALED)     # blob made for the other mode
    out = torch.full((1, 6, 6, 8), 1234567, dtype=torch.int32, device="cuda")
    wg.f2x2_conv2d_int8(_x(x, wg.NHWC), other, wg.NHWC, out=out)
    assert bool((out == 1234567).all())
    # a blob of the F(4x4,3x3) path is not accepted either
    p4 = wg.winograd_filter_transform(_g(g, wg.NHWC), wg.NHWC, wg.LOSSLESS)
    if p4.blob.numel() >= packed.blob.numel():
        wg.f2x2_conv2d_int8(_x(x, wg.NHWC), wg.F2x2PackedFilter(p4.blob, 8, 8, wg.LOSSLESS), wg.NHWC, out=out)
        assert bool((out == 1234567).all())


# ---- the paper's own setting: uint8 tensors with zero points (int9 values), Section 4.1 ------------------------

def _u8_case(N, C, K, H, W, zx, zw, seed):
    rng = np.random.default_rng(9000 + seed)
    xq = rng.integers(0, 256, (N, C, H, W)).astype(np.uint8)
    gq = rng.integers(0, 256, (K, C, 3, 3)).astype(np.uint8)
    return xq, gq, (xq.astype(np.int16) - zx), (gq.astype(np.int16) - zw)


def test_int9_filters_reach_the_printed_worst_case_table():
    """All taps 255 with zero point 0: the blob's limbs reassemble to 4, 6 and 9 times 255 at the corner, edge and
    centre entries — the 1020 / 1530 / 2295 of the printed table."""
    gq = np.full((2, 3, 3, 3), 255, np.uint8)
    packed = wg.f2x2_filter_transform(_dev(gq), wg.NCHW, wg.LOSSLESS, zero_point=0)
    planes, _ = wg.f2x2_debug_filter_operands(packed)
    planes = planes.cpu().numpy().astype(np.int64)
    Wt = (64 * planes[0::2] + planes[1::2]).reshape(4, 4, 2, 3)
    assert np.all(Wt[0, 0] == 1020) and np.all(Wt[0, 1] == 1530) and np.all(Wt[1, 1] == 2295) and np.all(Wt[3, 3] == 1020)
    assert np.array_equal(Wt[..., 0, 0], oracle.f2_filter_transform_i16(np.full((1, 1, 3, 3), 255, np.int16))[0, 0])


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("shape,zx,zw", [((1, 3, 5, 7, 9), 0, 255), ((2, 16, 16, 16, 16), 117, 131), ((1, 70, 33, 10, 6), 255, 0),
                                         ((1, 200, 72, 6, 10), 128, 128)])
def test_uint8_with_zero_points(shape, zx, zw, layout):
    N, C, K, H, W = shape
    xq, gq, x9, g9 = _u8_case(N, C, K, H, W, zx, zw, seed=C)
    xd = _dev(xq if layout == wg.NCHW else wl.to_nhwc(xq))
    gd = _dev(gq if layout == wg.NCHW else wl.to_krsc(gq))
    want = oracle.direct_conv2d_i16(x9, g9)
    y = wg.f2x2_conv2d_int8(xd, wg.f2x2_filter_transform(gd, layout, wg.LOSSLESS, zero_point=zw), layout, zero_point=zx)
    assert np.array_equal(_y(y, layout), want)
    packed = wg.f2x2_filter_transform(gd, layout, wg.SCALED, zero_point=zw)
    scaled, tab, _ = oracle.f2_scale_filters(oracle.f2_filter_transform_i16(g9), 127)
    planes, table = wg.f2x2_debug_filter_operands(packed)
    assert np.array_equal(planes.cpu().numpy().astype(np.int64), scaled.reshape(K, C, 16).transpose(2, 0, 1))
    y = wg.f2x2_conv2d_int8(xd, packed, layout, zero_point=zx)
    want_scaled, flags = oracle.f2_conv2d_i16(x9, g9, oracle.SCALED, 127)
    assert (flags & 4) == 0 and np.array_equal(_y(y, layout), want_scaled)


def test_uint8_extremes_at_the_largest_channel_count():
    C = wg.MAX_CHANNELS
    for xv, zx, gv, zw in ((255, 0, 255, 0), (0, 255, 255, 0), (0, 255, 0, 255)):
        xq = np.full((1, C, 4, 6), xv, np.uint8)
        gq = np.full((2, C, 3, 3), gv, np.uint8)
        gq[1] = 255 - gv
        y = wg.f2x2_conv2d_int8(_dev(wl.to_nhwc(xq)), wg.f2x2_filter_transform(_dev(wl.to_krsc(gq)), wg.NHWC, wg.LOSSLESS,
                                                                             zero_point=zw), wg.NHWC, zero_point=zx)
        assert np.array_equal(_y(y, wg.NHWC), oracle.direct_conv2d_i16(xq.astype(np.int16) - zx, gq.astype(np.int16) - zw))


def test_blobs_of_both_filter_transforms_serve_both_convolutions():
    """int8 activations with int9 filters and uint8 activations with int8 filters."""
    xq, gq, x9, g9 = _u8_case(1, 24, 20, 8, 8, 100, 140, seed=3)
    x8, g8 = wl.make_custom(1, 24, 20, 8, 8, seed=74)
    p9 = wg.f2x2_filter_transform(_dev(gq), wg.NCHW, wg.LOSSLESS, zero_point=140)
    p8 = wg.f2x2_filter_transform(_dev(g8), wg.NCHW, wg.LOSSLESS)
    y = wg.f2x2_conv2d_int8(_dev(x8), p9, wg.NCHW)
    assert np.array_equal(y.cpu().numpy(), oracle.direct_conv2d_i16(x8.astype(np.int16), g9))
    y = wg.f2x2_conv2d_int8(_dev(xq), p8, wg.NCHW, zero_point=100)
    assert np.array_equal(y.cpu().numpy(), oracle.direct_conv2d_i16(x9, g8.astype(np.int16)))


# ---- activations scaled per tile as well (the remark that closes Section 4.1) ---------------------------------

def _oracle_act_table(x):
    """[T, 16, 4] in the library's convention ("no scaling" stored as (0, 0, 1, 0))."""
    _, tab, _ = oracle.f2_scale_activations(oracle.f2_input_transform(x), 127)
    tab = tab.reshape(-1, 16, 4).copy()
    tab[tab[..., 0] == 0] = (0, 0, 1, 0)
    return tab


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("act", ["uniform", "relu"])
@pytest.mark.parametrize("shape", SHAPES)
def test_both_sides_scaled_equals_oracle(shape, act, layout):
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, act=act, wgt="gauss", seed=75)
    want, flags = oracle.f2_conv2d(x, g, oracle.BOTH_SCALED, 127)
    assert (flags & 4) == 0
    packed = wg.f2x2_filter_transform(_g(g, layout), layout, wg.SCALED)
    y, table = wg.f2x2_conv2d_int8_act_scaled(_x(x, layout), packed, layout, want_table=True)
    assert np.array_equal(table.cpu().numpy(), _oracle_act_table(x))
    assert np.array_equal(_y(y, layout), want)
    y2 = wg.f2x2_conv2d_int8_act_scaled(_x(x, layout), packed, layout)          # without the table export
    assert torch.equal(y, y2)


def test_both_sides_scaled_extremes_and_small_activations():
    """All-extreme activations at the largest channel count (every tile location at its largest magnitude), and
    activations small enough that no tile is scaled (the result is then the filter-scaled one)."""
    C = wg.MAX_CHANNELS
    for xv in (-128, 127):
        x = np.full((1, C, 5, 6), xv, np.int8)
        _, g = wl.make_custom(1, C, 3, 5, 6, wgt="uniform", seed=76)
        g[1] = 127
        want, flags = oracle.f2_conv2d(x, g, oracle.BOTH_SCALED, 127)
        assert (flags & 4) == 0
        packed = wg.f2x2_filter_transform(_g(g, wg.NHWC), wg.NHWC, wg.SCALED)
        y, table = wg.f2x2_conv2d_int8_act_scaled(_x(x, wg.NHWC), packed, wg.NHWC, want_table=True)
        assert np.array_equal(table.cpu().numpy(), _oracle_act_table(x))
        assert np.array_equal(_y(y, wg.NHWC), want)
    x = np.random.default_rng(77).integers(-31, 32, (2, 40, 9, 7)).astype(np.int8)
    _, g = wl.make_custom(2, 40, 24, 9, 7, wgt="gauss", seed=78)
    packed = wg.f2x2_filter_transform(_g(g, wg.NCHW), wg.NCHW, wg.SCALED)
    y, table = wg.f2x2_conv2d_int8_act_scaled(_dev(x), packed, wg.NCHW, want_table=True)
    assert bool((table[..., 0] == 0).all())
    assert torch.equal(y, wg.f2x2_conv2d_int8(_dev(x), packed, wg.NCHW))


@pytest.mark.parametrize("name", ["cfg2", "cfg4a", "cfg4b"])
def test_full_size_both_sides_scaled(name):
    """Benchmark configurations at full size in the launch configuration bench.py times; the oracle checks the first
    image and the last two."""
    x, g = wl.make_case(name)
    xd, gd = _x(x, wg.NHWC), _g(g, wg.NHWC)
    y = _y(wg.f2x2_conv2d_int8_act_scaled(xd, wg.f2x2_filter_transform(gd, wg.NHWC, wg.SCALED), wg.NHWC), wg.NHWC)
    for sl in (slice(0, 1), slice(x.shape[0] - 2, x.shape[0])):
        want, flags = oracle.f2_conv2d(x[sl], g, oracle.BOTH_SCALED, 127)
        assert (flags & 4) == 0
        assert np.array_equal(y[sl], want)


def test_act_scaled_rejects_a_lossless_blob():
    x, g = wl.make_custom(1, 8, 8, 6, 6, seed=79)
    packed = wg.f2x2_filter_transform(_g(g, wg.NHWC), wg.NHWC, wg.LOSSLESS)
    out = torch.full((1, 6, 6, 8), 1234567, dtype=torch.int32, device="cuda")
    wg.f2x2_conv2d_int8_act_scaled(_x(x, wg.NHWC), packed, wg.NHWC, out=out)
    assert bool((out == 1234567).all())


# ---- int8 epilogue: the requantisation that follows a quantised convolution (Section 4.4), inside the kernel ----

@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("mode", [wg.LOSSLESS, wg.SCALED])
@pytest.mark.parametrize("shape,relu,pool", [
    (shape, relu, pool)
    for shape in [(1, 4, 4, 4, 4), (2, 16, 16, 16, 16), (1, 70, 33, 10, 6), (3, 8, 100, 6, 14), (1, 130, 65, 8, 8), (1, 3, 5, 7, 9)]
    for relu, pool in [(True, False), (True, True), (False, False), (False, True)]
    if not (pool and ((shape[3] | shape[4]) & 1))])                       # pooling needs even H and W
def test_int8_epilogue_equals_oracle_requantisation(shape, relu, pool, mode, layout):
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, act="relu", wgt="gauss", seed=90)
    if mode == wg.LOSSLESS:
        want32 = oracle.direct_conv2d(x, g)
    else:
        want32, flags = oracle.f2_conv2d(x, g, oracle.SCALED, 127)
        assert (flags & 4) == 0
    shift = max(0, int(np.abs(want32).max()).bit_length() - 7)
    want = oracle.requant_relu_pool(want32, shift, relu, pool)
    packed = wg.f2x2_filter_transform(_g(g, layout), layout, mode)
    Ho, Wo = (H // 2, W // 2) if pool else (H, W)
    out = torch.full((N, K, Ho, Wo) if layout == wg.NCHW else (N, Ho, Wo, K), 77, dtype=torch.int8, device="cuda")
    wg.f2x2_conv2d_int8_requant(_x(x, layout), packed, shift, relu, pool, layout, out=out)
    got = out.cpu().numpy()
    assert np.array_equal(got if layout == wg.NCHW else wl.from_nhwc(got), want)
    assert want.max() > 0 and (relu or pool or want.min() < 0)      # the case exercises both signs where it can


def test_int8_epilogue_full_size_cfg3():
    x, g = wl.make_case("cfg3")
    xd, gd = _x(x, wg.NHWC), _g(g, wg.NHWC)
    packed = wg.f2x2_filter_transform(gd, wg.NHWC, wg.LOSSLESS)
    y32 = wg.f2x2_conv2d_int8(xd, packed, wg.NHWC)
    shift = max(0, int(y32.abs().max().item()).bit_length() - 7)
    q = wg.f2x2_conv2d_int8_requant(xd, packed, shift, True, True, wg.NHWC)
    assert torch.equal(q, wg.requant_relu_pool_int8(y32, shift, True, True, wg.NHWC))
    want = oracle.requant_relu_pool(oracle.direct_conv2d(x[:1], g), shift, True, True)
    assert np.array_equal(wl.from_nhwc(q[:1].cpu().numpy()), want)
