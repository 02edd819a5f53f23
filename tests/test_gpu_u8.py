"""GPU parity of the complex F(4x4,3x3) path on the quantised tensors of Section 4.1 (uint8 bytes with zero points,
i.e. int9 values), through winograd_filter_transform_u8 / winograd_conv2d_u8, bit for bit against the CPU oracle's
16-bit functions."""
import numpy as np
import pytest
import torch

import oracle
import paper_1901_01965_amd as wg
from paper_1901_01965_amd import workloads as wl

pytestmark = pytest.mark.gpu

R = (0, 1, 2, 5)
ENTRIES = [(r, c) for r in R for c in R] + [(r, 3) for r in R] + [(3, c) for c in R] + [(3, 3), (3, 4)]
LAYOUTS = [wg.NHWC, wg.NCHW]


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _x(x, layout):
    return _dev(x if layout == wg.NCHW else wl.to_nhwc(x))


def _g(g, layout):
    return _dev(g if layout == wg.NCHW else wl.to_krsc(g))


def _y(y, layout):
    y = y.cpu().numpy()
    return y if layout == wg.NCHW else wl.from_nhwc(y)


def _case(N, C, K, H, W, zx, zw, seed):
    rng = np.random.default_rng(4300 + seed)
    xq = rng.integers(0, 256, (N, C, H, W)).astype(np.uint8)
    gq = rng.integers(0, 256, (K, C, 3, 3)).astype(np.uint8)
    gq[0] = 255          # a whole filter and single taps at both ends of the byte range
    gq[-1, :, 1, 1] = 0
    xq[0, :, : max(1, H // 2)] = 255
    xq[0, :, :, :1] = 0
    return xq, gq, (xq.astype(np.int16) - zx), (gq.astype(np.int16) - zw)


def test_int9_filters_reach_thirteen_bits_in_the_blob():
    """All taps 255 with zero point 0: the limbs in the blob reassemble to 16 * 255 = 4080 at the corner entries,
    and the scaled blob holds them as 15/512 of that."""
    gq = np.full((2, 5, 3, 3), 255, np.uint8)
    gq[1] = 0
    g9 = gq.astype(np.int16) - 0
    packed = wg.winograd_filter_transform_u8(_dev(gq), 0, wg.NCHW, wg.LOSSLESS)
    packed.check()
    planes, _ = wg.debug_filter_operands(packed)
    planes = planes.cpu().numpy().astype(np.int64)
    Wt = oracle.filter_transform_i16(g9)
    vals = 64 * planes[0::3] + planes[1::3]
    assert vals[0].max() == 4080 and np.array_equal(vals[0], Wt[:, :, 0, 0, 0])
    assert np.array_equal(planes[2::3], planes[0::3] + planes[1::3])
    packed = wg.winograd_filter_transform_u8(_dev(gq), 0, wg.NCHW, wg.SCALED)
    planes, table = wg.debug_filter_operands(packed)
    assert table.cpu().numpy()[0, 0].tolist() == [15, 9, 137, 2]
    assert planes.cpu().numpy()[0, 0, 0] == (4080 * 15 + 256) >> 9 == 120


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("kc,zw", [((4, 4), 0), ((5, 3), 255), ((64, 64), 128), ((33, 70), 77), ((40, 229), 200)])
def test_filter_blobs_equal_the_oracles_filters(kc, zw, layout):
    K, C = kc
    _, gq, _, g9 = _case(1, C, K, 4, 4, 0, zw, seed=K)
    Wt = oracle.filter_transform_i16(g9)
    planes, table = wg.debug_filter_operands(wg.winograd_filter_transform_u8(_g(gq, layout), zw, layout, wg.LOSSLESS))
    planes = planes.cpu().numpy().astype(np.int64)
    vals = [Wt[:, :, r, c, 0] for (r, c) in ENTRIES[:16]]
    for (r, c) in ENTRIES[16:]:
        vals += [Wt[:, :, r, c, 0], Wt[:, :, r, c, 1], Wt[:, :, r, c, 0] + Wt[:, :, r, c, 1]]
    vals = np.stack(vals)
    assert np.array_equal(planes[0::3], vals >> 6) and np.array_equal(planes[1::3], vals & 63)
    assert np.abs(planes).max() <= 127 and (table.cpu().numpy() == np.array([0, 0, 1, 0])).all()
    planes, table = wg.debug_filter_operands(wg.winograd_filter_transform_u8(_g(gq, layout), zw, layout, wg.SCALED))
    Ws, tab, mx = oracle.scale_filters(Wt, 127)
    want = [Ws[:, :, r, c, 0] for (r, c) in ENTRIES[:16]]
    for (r, c) in ENTRIES[16:]:
        want += [Ws[:, :, r, c, 0], Ws[:, :, r, c, 1], -Ws[:, :, r, c, 1]]
    assert np.array_equal(planes.cpu().numpy().astype(np.int64), np.stack(want))
    assert np.array_equal(table.cpu().numpy(), np.stack([tab[:, r, c] for (r, c) in ENTRIES], axis=1))


SHAPES = [  # (N, C, K, H, W), zero point of x, zero point of w
    ((1, 1, 1, 1, 1), 3, 250),
    ((1, 3, 5, 7, 9), 0, 255),          # byte loads, ragged tiles
    ((2, 16, 16, 16, 16), 117, 131),    # 4-byte loads when channels-last
    ((1, 70, 33, 10, 6), 255, 0),       # two channel blocks, C % 4 != 0
    ((3, 8, 100, 5, 13), 128, 128),     # ragged last filter block
    ((1, 200, 72, 6, 10), 1, 254),      # four channel blocks
    ((1, 229, 40, 9, 9), 128, 127),     # the largest channel count
    ((2, 64, 64, 56, 56), 128, 128),    # the quoted layer's shape at batch 2
]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("shape,zx,zw", SHAPES)
def test_uint8_with_zero_points(shape, zx, zw, layout):
    N, C, K, H, W = shape
    xq, gq, x9, g9 = _case(N, C, K, H, W, zx, zw, seed=C + K)
    xd, gd = _x(xq, layout), _g(gq, layout)
    out = torch.full((N, K, H, W) if layout == wg.NCHW else (N, H, W, K), 13579, dtype=torch.int32, device="cuda")
    wg.winograd_conv2d_u8(xd, zx, wg.winograd_filter_transform_u8(gd, zw, layout, wg.LOSSLESS), layout, out=out)
    assert np.array_equal(_y(out, layout), oracle.direct_conv2d_i16(x9, g9))
    want, flags = oracle.winograd_conv2d_i16(x9, g9, oracle.SCALED, 127)
    assert (flags & 5) == 0
    y = wg.winograd_conv2d_u8(xd, zx, wg.winograd_filter_transform_u8(gd, zw, layout, wg.SCALED), layout)
    assert np.array_equal(_y(y, layout), want)


@pytest.mark.parametrize("layout", LAYOUTS)
def test_extreme_bytes_and_zero_points_at_229_channels(layout):
    """|x| = |w| = 255 everywhere: interior outputs are +-9 * 229 * 255^2, whose sixteenfold still fits int32
    (the reason for the channel limit); every limb and the padding selection at their extremes."""
    C = wg.MAX_CHANNELS_U8
    for xv, zx, gv, zw in ((255, 0, 255, 0), (0, 255, 255, 0), (255, 0, 0, 255), (0, 255, 0, 255)):
        xq = np.full((1, C, 12, 8), xv, np.uint8)
        gq = np.full((3, C, 3, 3), gv, np.uint8)
        gq[1] = 255 - gv                       # filters equal to the zero point: all zero
        gq[2, :, ::2, ::2] = 255 - gv
        x9, g9 = xq.astype(np.int16) - zx, gq.astype(np.int16) - zw
        want = oracle.direct_conv2d_i16(x9, g9)
        assert np.abs(want.astype(np.int64)).max() == 9 * C * 255 * 255 and 16 * 9 * C * 255 * 255 < 2 ** 31
        y = wg.winograd_conv2d_u8(_x(xq, layout), zx, wg.winograd_filter_transform_u8(_g(gq, layout), zw, layout, wg.LOSSLESS),
                                  layout)
        assert np.array_equal(_y(y, layout), want)


def test_signed_int8_filters_enter_as_bytes_with_zero_point_128():
    x8, g8 = wl.make_custom(1, 24, 20, 8, 8, seed=74)
    xq = np.random.default_rng(5).integers(0, 256, x8.shape).astype(np.uint8)
    gq = (g8.astype(np.int16) + 128).astype(np.uint8)
    y = wg.winograd_conv2d_u8(_dev(xq), 90, wg.winograd_filter_transform_u8(_dev(gq), 128, wg.NCHW, wg.LOSSLESS), wg.NCHW)
    assert np.array_equal(y.cpu().numpy(), oracle.direct_conv2d_i16(xq.astype(np.int16) - 90, g8.astype(np.int16)))


def test_limits_and_mismatches():
    lib = wg.load_library()
    C = wg.MAX_CHANNELS_U8 + 1
    gq = torch.zeros((4, C, 3, 3), dtype=torch.uint8, device="cuda")
    with pytest.raises(wg.WinogradError) as e:
        wg.winograd_filter_transform_u8(gq, 0, wg.NCHW, wg.LOSSLESS)
    assert e.value.status == -2
    blob = torch.zeros(wg.packed_filter_bytes(4, C, wg.LOSSLESS), dtype=torch.uint8, device="cuda")
    xq = torch.zeros((1, C, 4, 4), dtype=torch.uint8, device="cuda")
    y = torch.zeros((1, 4, 4, 4), dtype=torch.int32, device="cuda")
    assert lib.winograd_conv2d_u8(xq.data_ptr(), 0, blob.data_ptr(), y.data_ptr(), 1, C, 4, 4, 4, wg.NCHW, wg.LOSSLESS, None) == -2
    assert lib.winograd_conv2d_u8(xq.data_ptr(), 256, blob.data_ptr(), y.data_ptr(), 1, 8, 4, 4, 4, wg.NCHW, wg.LOSSLESS, None) == -1
    assert lib.winograd_filter_transform_u8(gq.data_ptr(), -1, 4, 8, wg.NCHW, wg.LOSSLESS, blob.data_ptr(), blob.numel(), None) == -1
    # the two kinds of blob do not mix: the binding says so, and the kernels leave the output untouched
    x8, g8 = wl.make_custom(1, 8, 6, 8, 8, seed=42)
    p8 = wg.winograd_filter_transform(_dev(g8), wg.NCHW, wg.LOSSLESS)
    p9 = wg.winograd_filter_transform_u8(_dev(g8.view(np.uint8)), 0, wg.NCHW, wg.LOSSLESS)
    with pytest.raises(TypeError):
        wg.winograd_conv2d_u8(_dev(x8.view(np.uint8)), 0, p8, wg.NCHW)
    with pytest.raises(TypeError):
        wg.winograd_conv2d_int8(_dev(x8), p9, wg.NCHW)
    out = torch.full((1, 6, 8, 8), 24680, dtype=torch.int32, device="cuda")
    wg.winograd_conv2d_u8(_dev(x8.view(np.uint8)), 0, wg.PackedFilterU8(p8.blob, p8.K, p8.C, p8.mode), wg.NCHW, out=out)
    assert (out == 24680).all()
    wg.winograd_conv2d_int8(_dev(x8), wg.PackedFilter(p9.blob, p9.K, p9.C, p9.mode), wg.NCHW, out=out)
    assert (out == 24680).all()
    wg.force_path(wg.STAGED)
    try:
        wg.winograd_conv2d_int8(_dev(x8), wg.PackedFilter(p9.blob, p9.K, p9.C, p9.mode), wg.NCHW, out=out)
    finally:
        wg.force_path(wg.AUTO)
    assert (out == 24680).all()
