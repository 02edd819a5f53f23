"""GPU parity of the role-specialised kernel with eight product waves (twelve waves and 64 filters per workgroup: four
waves transform, product wave pw owns filter block pw % 4 and half pw / 4 of the free entries and keeps 18 joined channel
sums; the two 32-filter halves stage and store side by side), scaled mode, forced through the test hook on shapes the
library would give to other kernels as well: bit for bit against the CPU oracle's scaled mode."""
import numpy as np
import pytest
import torch

import oracle
import paper_1901_01965_amd as wg
from paper_1901_01965_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def eight_product_waves():
    wg.scaled_variant(1)
    yield
    wg.scaled_variant(0)


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _want(x, g, mode=None):
    if mode == wg.LOSSLESS:
        return oracle.direct_conv2d(x, g)
    want, flags = oracle.winograd_conv2d(x, g, oracle.SCALED, 127)
    assert (flags & 5) == 0
    return want


SHAPES = [  # N, C, K, H, W (channels-last, C % 4 == 0, C > 4)
    (2, 16, 16, 16, 16),      # 16-byte patch transfer, one channel block, filters padded to 64
    (1, 8, 100, 5, 13),       # 4-byte pixel loads, ragged tiles, ragged last filter block
    (2, 64, 64, 12, 12),      # a full channel block
    (1, 32, 48, 30, 18),      # several tile blocks, ragged last one
    (1, 200, 40, 9, 9),       # four channel blocks, the last with 8 channels, 4-byte loads
    (2, 80, 72, 14, 14),      # two channel blocks, the last with 16 channels, 16-byte transfer
    (1, 132, 36, 26, 10),     # three channel blocks, 4-byte loads
    (1, 16, 72, 131, 131),    # many tile blocks (more workgroups than compute units)
    (3, 20, 6, 7, 9),         # K % 4 != 0: element-wise stores
    (1, 64, 33, 8, 8),        # K odd
    (4, 512, 64, 7, 7),       # eight channel blocks, partial tiles (the deepest configuration's shape)
]


@pytest.mark.parametrize("mode", [wg.SCALED, wg.LOSSLESS])
@pytest.mark.parametrize("act", ["relu", "uniform"])
@pytest.mark.parametrize("shape", SHAPES)
def test_equals_oracle(shape, act, mode):
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, act=act, wgt="uniform" if act == "uniform" else "gauss", seed=191)
    if act == "uniform":
        g[0] = -128                       # Winograd-domain magnitude 2048: the factor's p = 8
        x[0, :, : max(1, H // 2)] = -128
    packed = wg.winograd_filter_transform(_dev(wl.to_krsc(g)), wg.NHWC, mode)
    out = torch.full((N, H, W, K), 1357911, dtype=torch.int32, device="cuda")
    wg.winograd_conv2d_int8(_dev(wl.to_nhwc(x)), packed, wg.NHWC, out=out)
    assert np.array_equal(wl.from_nhwc(out.cpu().numpy()), _want(x, g, mode))


@pytest.mark.parametrize("xv", [-128, 127])
def test_extreme_activations_and_most_channels(xv):
    """Every activation limb at its extreme over 14 channel blocks: the resident limb accumulators hold
    sums of up to 896 * 9 ... products without overflow, and 256 high + low is exact."""
    C = wg.MAX_CHANNELS
    x = np.full((1, C, 12, 8), xv, np.int8)
    _, g = wl.make_custom(1, C, 10, 12, 8, wgt="uniform", seed=192)
    g[0], g[1] = -128, 127
    packed = wg.winograd_filter_transform(_dev(wl.to_krsc(g)), wg.NHWC, wg.SCALED)
    y = wg.winograd_conv2d_int8(_dev(wl.to_nhwc(x)), packed, wg.NHWC)
    assert np.array_equal(wl.from_nhwc(y.cpu().numpy()), _want(x, g))


@pytest.mark.parametrize("offset", [0, 4, 8])
def test_input_alignment_selects_equivalent_load_paths(offset):
    N, C, K, H, W = 2, 80, 40, 11, 13
    x, g = wl.make_custom(N, C, K, H, W, seed=193)
    xs = wl.to_nhwc(x)
    buf = torch.zeros(xs.size + 16, dtype=torch.int8, device="cuda")
    xd = buf[offset:offset + xs.size].view(N, H, W, C)
    xd.copy_(torch.from_numpy(xs))
    assert xd.data_ptr() % 16 == offset
    packed = wg.winograd_filter_transform(_dev(wl.to_krsc(g)), wg.NHWC, wg.SCALED)
    y = wg.winograd_conv2d_int8(xd, packed, wg.NHWC)
    assert np.array_equal(wl.from_nhwc(y.cpu().numpy()), _want(x, g))


def test_output_canaries_and_unaligned_output():
    N, C, K, H, W = 1, 16, 8, 7, 5
    x, g = wl.make_custom(N, C, K, H, W, seed=194)
    packed = wg.winograd_filter_transform(_dev(wl.to_krsc(g)), wg.NHWC, wg.SCALED)
    n = N * H * W * K
    for lead in (64, 65):
        buf = torch.full((lead + n + 64,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
        out = buf[lead:lead + n].view(N, H, W, K)
        wg.winograd_conv2d_int8(_dev(wl.to_nhwc(x)), packed, wg.NHWC, out=out)
        assert np.array_equal(wl.from_nhwc(out.cpu().numpy()), _want(x, g))
        assert (buf[:lead] == 0x5A5A5A5A).all() and (buf[-64:] == 0x5A5A5A5A).all()


@pytest.mark.parametrize("shape", [(2, 16, 32, 8, 12), (2, 20, 36, 10, 6), (1, 64, 7, 4, 4), (3, 32, 64, 18, 22), (1, 132, 68, 8, 8),
                                   (1, 16, 6, 7, 9), (2, 256, 64, 14, 14)])
def test_int8_epilogue_equals_oracle_conv_then_requantisation(shape):
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, seed=195)
    want32 = _want(x, g)
    top = max(1, int(np.abs(want32).max()))
    packed = wg.winograd_filter_transform(_dev(wl.to_krsc(g)), wg.NHWC, wg.SCALED)
    xd = _dev(wl.to_nhwc(x))
    for shift in sorted({0, max(0, top.bit_length() - 8), max(0, top.bit_length() - 6)}):
        for relu in (True, False):
            for pool in (False, True):
                if pool and (H % 2 or W % 2):
                    continue
                Ho, Wo = (H // 2, W // 2) if pool else (H, W)
                out = torch.full((N, Ho, Wo, K), 77, dtype=torch.int8, device="cuda")
                wg.winograd_conv2d_int8_requant(xd, packed, shift, relu, pool, wg.NHWC, out=out)
                assert np.array_equal(wl.from_nhwc(out.cpu().numpy()), oracle.requant_relu_pool(want32, shift, relu, pool)), (
                    shift, relu, pool)


@pytest.mark.parametrize("name", ["cfg3", "cfg4a", "cfg4b"])
def test_full_size_configurations_agree_with_the_other_forms_and_the_oracle(name):
    x, g = wl.make_case(name)
    xd, gd = _dev(wl.to_nhwc(x)), _dev(wl.to_krsc(g))
    packed = wg.winograd_filter_transform(gd, wg.NHWC, wg.SCALED)
    y_eight = wg.winograd_conv2d_int8(xd, packed, wg.NHWC)
    wg.scaled_variant(2)
    y_other = wg.winograd_conv2d_int8(xd, packed, wg.NHWC)
    assert torch.equal(y_eight, y_other)
    got = wl.from_nhwc(y_eight.cpu().numpy())
    for sl in (slice(0, 1), slice(x.shape[0] - 2, x.shape[0])):
        assert np.array_equal(got[sl], _want(x[sl], g))
