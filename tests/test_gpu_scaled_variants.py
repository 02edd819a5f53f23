"""GPU parity of every variant of the single-kernel path on full-range and extreme int8 data, int32 output,
bit for bit against the CPU oracle.

The other parity files feed the scaled mode post-ReLU activations; here the activations cover all of
[-128, 127], or are all -128 / all 127 (the transformed value at entry (1,1) of an interior tile is then
16 * (-128) = -2048, the most negative 12-bit operand, and every limb split sees its extreme), and the filters
contain -128 taps (a Winograd-domain magnitude of 2048 needs the scale factor's p = 8).  Each case names the
kernel variant its shape (or the test hook) selects."""
import numpy as np
import pytest
import torch

import oracle
import paper_1901_01965_amd as wg
from paper_1901_01965_amd import workloads as wl

pytestmark = pytest.mark.gpu

# (variant, layout, (N, C, K, H, W), streaming workgroups per filter block or 0)
CASES = [
    ("monolithic, byte loads, one channel block", wg.NCHW, (2, 20, 36, 13, 14), 0),
    ("monolithic, byte loads, channel sums", wg.NCHW, (1, 70, 33, 12, 13), 0),
    ("monolithic, byte loads, channels-last, C % 4 != 0", wg.NHWC, (1, 70, 33, 12, 13), 0),
    ("monolithic, byte loads, channels-last, six channels", wg.NHWC, (2, 6, 20, 12, 16), 0),
    ("monolithic, 4-byte loads", wg.NHWC, (2, 20, 36, 13, 14), 0),
    ("monolithic, 16-byte direct transfer", wg.NHWC, (2, 32, 40, 14, 13), 0),
    ("monolithic, 16-byte direct transfer, 64 channels", wg.NHWC, (1, 64, 64, 16, 12), 0),
    ("64 filters per workgroup, one channel block", wg.NHWC, (1, 16, 72, 131, 131), 0),
    ("64 filters per workgroup, two channel blocks", wg.NHWC, (2, 80, 128, 92, 92), 0),
    ("role-specialised, three channel blocks", wg.NHWC, (1, 132, 36, 26, 10), 0),
    ("role-specialised, two channel blocks", wg.NHWC, (2, 80, 72, 14, 14), 0),
    ("role-specialised, four channel blocks", wg.NHWC, (1, 200, 32, 12, 12), 0),
    ("streaming, one channel block", wg.NHWC, (3, 64, 40, 18, 22), 4),
    ("streaming, two channel blocks", wg.NHWC, (2, 80, 72, 14, 14), 2),
    ("streaming, three channel blocks, ragged", wg.NHWC, (1, 132, 36, 26, 10), 5),
    ("streaming, one tile block per workgroup", wg.NHWC, (1, 16, 32, 16, 16), 1),
]


def _inputs(shape, act):
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, act="uniform", wgt="uniform", seed=71)
    if act == "min":
        x[:] = -128
    elif act == "max":
        x[:] = 127
    # -128 taps: a whole filter (its corner entries reach 16 * 128 = 2048), one tap of another, and a filter
    # that is +-127 / -128 in a checkerboard, so that the complex entries are large as well
    g[0] = -128
    g[1 % K, :, 0, 0] = -128
    g[2 % K] = np.where((np.indices((3, 3)).sum(0) % 2 == 0), -128, 127).astype(np.int8)
    return x, g


@pytest.mark.parametrize("mode", [wg.SCALED, wg.LOSSLESS])
@pytest.mark.parametrize("act", ["uniform", "min", "max"])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_single_kernel_variants_on_full_range_data(case, act, mode):
    name, layout, shape, slots = case
    N, C, K, H, W = shape
    x, g = _inputs(shape, act)
    if mode == wg.LOSSLESS:
        want = oracle.direct_conv2d(x, g)
    else:
        want, flags = oracle.winograd_conv2d(x, g, oracle.SCALED, 127)
        assert (flags & 5) == 0
        if act != "uniform":
            # the data drive the operands to their extremes: check that on the oracle's own arrays
            D11 = oracle.input_transform(x[:1])[..., 1, 1, 0]
            assert (D11.min() == -2048) if act == "min" else (D11.max() == 2032)
        _, tab, mx = oracle.scale_filters(oracle.filter_transform(g), 127)
        assert mx.max() == 2048 and tab[..., 1].max() == 8
    xd = torch.from_numpy(x if layout == wg.NCHW else wl.to_nhwc(x)).cuda()
    gd = torch.from_numpy(g if layout == wg.NCHW else wl.to_krsc(g)).cuda()
    packed = wg.winograd_filter_transform(gd, layout, mode)
    wg.stream_workgroups(slots)
    try:
        y = wg.winograd_conv2d_int8(xd, packed, layout).cpu().numpy()
    finally:
        wg.stream_workgroups(0)
    got = y if layout == wg.NCHW else wl.from_nhwc(y)
    assert np.array_equal(got, want), name


def test_binding_rejects_blobs_and_outputs_that_do_not_fit():
    """A blob packed for another channel count or another algorithm, or an output tensor of the wrong shape or
    type, is an error in the binding (the kernels could only leave the output untouched)."""
    x, g = wl.make_custom(1, 8, 6, 8, 8, seed=42)
    xd = torch.from_numpy(wl.to_nhwc(x)).cuda()
    gd = torch.from_numpy(wl.to_krsc(g)).cuda()
    packed = wg.winograd_filter_transform(gd, wg.NHWC, wg.LOSSLESS)
    other_c = wg.winograd_filter_transform(torch.from_numpy(wl.to_krsc(g[:, :4])).cuda(), wg.NHWC, wg.LOSSLESS)
    f2 = wg.f2x2_filter_transform(gd, wg.NHWC, wg.LOSSLESS)
    with pytest.raises(ValueError):
        wg.winograd_conv2d_int8(xd, other_c, wg.NHWC)
    with pytest.raises(TypeError):
        wg.winograd_conv2d_int8(xd, f2, wg.NHWC)
    with pytest.raises(TypeError):
        wg.f2x2_conv2d_int8(xd, packed, wg.NHWC)
    with pytest.raises(ValueError):
        wg.winograd_conv2d_int8(xd, packed, wg.NHWC, out=torch.empty((1, 8, 8, 5), dtype=torch.int32, device="cuda"))
    with pytest.raises(TypeError):
        wg.winograd_conv2d_int8(xd, packed, wg.NHWC, out=torch.empty((1, 8, 8, 6), dtype=torch.int8, device="cuda"))
    with pytest.raises(ValueError):
        wg.winograd_conv2d_int8_requant(xd, packed, 5, True, True, wg.NHWC,
                                        out=torch.empty((1, 8, 8, 6), dtype=torch.int8, device="cuda"))
    with pytest.raises(ValueError):
        wg.direct_conv2d_int8(xd, torch.from_numpy(wl.to_krsc(g[:, :4])).cuda(), wg.NHWC)
    y = wg.winograd_conv2d_int8(xd, packed, wg.NHWC)
    assert np.array_equal(wl.from_nhwc(y.cpu().numpy()), oracle.direct_conv2d(x, g))


@pytest.mark.parametrize("mode", [wg.LOSSLESS, wg.SCALED])
@pytest.mark.parametrize("shift", [20, 23, 27, 28, 31])
def test_narrow_input_int8_epilogue_with_large_shifts(shift, mode):
    """First-layer kernel (C <= 4): it folds the final division by 16 and the requantisation shift into one
    shift; every shift the entry point accepts must still equal the two-step definition."""
    x, g = wl.make_custom(1, 3, 70, 12, 8, seed=73)
    g[0] = -128
    x[0, :, :6] = -128
    want32 = oracle.direct_conv2d(x, g) if mode == wg.LOSSLESS else oracle.winograd_conv2d(x, g, oracle.SCALED)[0]
    xd = torch.from_numpy(wl.to_nhwc(x)).cuda()
    packed = wg.winograd_filter_transform(torch.from_numpy(wl.to_krsc(g)).cuda(), wg.NHWC, mode)
    for relu in (False, True):
        for pool in (False, True):
            got = wg.winograd_conv2d_int8_requant(xd, packed, shift, relu, pool, wg.NHWC)
            assert np.array_equal(wl.from_nhwc(got.cpu().numpy()), oracle.requant_relu_pool(want32, shift, relu, pool))
