"""GPU parity of the streaming kernel's 64-filter form (each product wave owns every entry of 16 filters; a tile block's
outputs staged as one finished copy per 32 filters), forced through the test hooks on small shapes: bit for bit against
the CPU oracle, int32 and int8 outputs.  The form serves lossless mode with any number of channel blocks and scaled
mode with one; the scaled cases with more channel blocks run the 32-filter form and check that the hook leaves them
right."""
import numpy as np
import pytest
import torch

import oracle
import paper_1901_01965_amd as wg
from paper_1901_01965_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def wide_stream():
    wg.stream_variant(1)
    wg.scaled_variant(2)      # keep the role-specialised (non-streaming) form with eight product waves out of the way
    yield
    wg.stream_variant(0)
    wg.scaled_variant(0)
    wg.stream_workgroups(0)


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _want(x, g, mode):
    if mode == wg.LOSSLESS:
        return oracle.direct_conv2d(x, g)
    want, flags = oracle.winograd_conv2d(x, g, oracle.SCALED, 127)
    assert (flags & 5) == 0
    return want


CASES = [  # (N, C, K, H, W), workgroups per filter block
    ((3, 64, 40, 18, 22), 4),       # one channel block, several tile blocks per workgroup, ragged tiles
    ((2, 80, 72, 14, 14), 2),       # two channel blocks, K padded to 128: two 64-filter groups
    ((1, 132, 36, 26, 10), 5),      # three channel blocks, ragged last range
    ((1, 16, 32, 16, 16), 1),       # one tile block per workgroup
    ((2, 64, 64, 56, 56), 7),       # the quoted layer's shape at batch 2, 14 tile blocks per workgroup
    ((1, 256, 128, 20, 12), 3),     # four channel blocks
    ((1, 16, 64, 9, 9), 40),        # more workgroups than tile blocks
]


@pytest.mark.parametrize("mode", [wg.SCALED, wg.LOSSLESS])
@pytest.mark.parametrize("act", ["relu", "uniform"])
@pytest.mark.parametrize("case", CASES)
def test_equals_oracle(case, act, mode):
    (N, C, K, H, W), slots = case
    x, g = wl.make_custom(N, C, K, H, W, act=act, wgt="uniform" if act == "uniform" else "gauss", seed=291)
    if act == "uniform":
        g[0] = -128
        x[0, :, : max(1, H // 2)] = -128
    packed = wg.winograd_filter_transform(_dev(wl.to_krsc(g)), wg.NHWC, mode)
    out = torch.full((N, H, W, K), 1357911, dtype=torch.int32, device="cuda")
    wg.stream_workgroups(slots)
    wg.winograd_conv2d_int8(_dev(wl.to_nhwc(x)), packed, wg.NHWC, out=out)
    assert np.array_equal(wl.from_nhwc(out.cpu().numpy()), _want(x, g, mode))


@pytest.mark.parametrize("mode", [wg.SCALED, wg.LOSSLESS])
@pytest.mark.parametrize("case", [((2, 16, 32, 8, 12), 2), ((3, 32, 64, 18, 22), 3), ((1, 132, 68, 8, 8), 1), ((2, 256, 64, 14, 14), 2)])
def test_int8_epilogue_equals_oracle_conv_then_requantisation(case, mode):
    (N, C, K, H, W), slots = case
    x, g = wl.make_custom(N, C, K, H, W, seed=295)
    want32 = _want(x, g, mode)
    top = max(1, int(np.abs(want32).max()))
    packed = wg.winograd_filter_transform(_dev(wl.to_krsc(g)), wg.NHWC, mode)
    xd = _dev(wl.to_nhwc(x))
    wg.stream_workgroups(slots)
    for shift in sorted({0, max(0, top.bit_length() - 8), max(0, top.bit_length() - 6)}):
        for relu in (True, False):
            for pool in (False, True):
                Ho, Wo = (H // 2, W // 2) if pool else (H, W)
                out = torch.full((N, Ho, Wo, K), 77, dtype=torch.int8, device="cuda")
                wg.winograd_conv2d_int8_requant(xd, packed, shift, relu, pool, wg.NHWC, out=out)
                assert np.array_equal(wl.from_nhwc(out.cpu().numpy()), oracle.requant_relu_pool(want32, shift, relu, pool)), (
                    shift, relu, pool)


def test_extreme_activations_and_most_channels():
    C = wg.MAX_CHANNELS
    for xv in (-128, 127):
        x = np.full((1, C, 12, 8), xv, np.int8)
        _, g = wl.make_custom(1, C, 12, 12, 8, wgt="uniform", seed=292)
        g[0], g[1] = -128, 127
        for mode in (wg.SCALED, wg.LOSSLESS):
            packed = wg.winograd_filter_transform(_dev(wl.to_krsc(g)), wg.NHWC, mode)
            wg.stream_workgroups(2)
            y = wg.winograd_conv2d_int8(_dev(wl.to_nhwc(x)), packed, wg.NHWC)
            assert np.array_equal(wl.from_nhwc(y.cpu().numpy()), _want(x, g, mode))


@pytest.mark.parametrize("N", [8, 12, 40])
def test_library_choice_on_the_quoted_layer_at_small_and_medium_batch(N):
    """No hooks: the quoted layer's shape (64 channels, 64 filters, 56x56) at batches around the points where the library
    changes kernels.  N = 8: one round of 32-filter workgroups (lossless: limb-pair kernel; scaled: the streaming kernel's
    32-filter form, one tile block per workgroup).  N = 12: the 32-filter grid exceeds one round, the 64-filter grid does
    not (lossless: this file's 64-filter streaming form; scaled: the role-specialised kernel with eight product waves).
    N = 40: both exceed it (64-filter streaming form in both modes).  Lossless equals the direct kernel everywhere; both
    modes equal the oracle on the first and the last image."""
    wg.stream_variant(0)
    wg.scaled_variant(0)
    C, K, H, W = 64, 64, 56, 56
    x, g = wl.make_custom(N, C, K, H, W, act="relu", wgt="gauss", seed=296)
    xd, gd = _dev(wl.to_nhwc(x)), _dev(wl.to_krsc(g))
    y = wg.winograd_conv2d_int8(xd, wg.winograd_filter_transform(gd, wg.NHWC, wg.LOSSLESS), wg.NHWC)
    assert torch.equal(y, wg.direct_conv2d_int8(xd, gd, wg.NHWC))
    ys = wg.winograd_conv2d_int8(xd, wg.winograd_filter_transform(gd, wg.NHWC, wg.SCALED), wg.NHWC)
    for sl in (slice(0, 1), slice(N - 1, N)):
        assert np.array_equal(wl.from_nhwc(y[sl].cpu().numpy()), oracle.direct_conv2d(x[sl], g))
        assert np.array_equal(wl.from_nhwc(ys[sl].cpu().numpy()), _want(x[sl], g, wg.SCALED))
