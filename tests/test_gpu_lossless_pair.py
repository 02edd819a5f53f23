"""GPU parity of the limb-pair form of the lossless single-kernel path (eight waves per 16 tiles x 32 filters; the filter
operand of the matrix cores carries both int8 limbs of eight filters), forced through the test hook on shapes the
library would give to other kernels as well: bit for bit against the CPU oracle's direct convolution."""
import numpy as np
import pytest
import torch

import oracle
import paper_1901_01965_amd as wg
from paper_1901_01965_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def pair_form():
    wg.lossless_variant(1)
    yield
    wg.lossless_variant(0)


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


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
]


@pytest.mark.parametrize("shape", SHAPES)
def test_lossless_equals_oracle_direct(shape):
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, seed=91)
    g[0] = -128
    x[0, :, : H // 2] = -128
    packed = wg.winograd_filter_transform(_dev(wl.to_krsc(g)), wg.NHWC, wg.LOSSLESS)
    out = torch.full((N, H, W, K), 1357911, dtype=torch.int32, device="cuda")
    wg.winograd_conv2d_int8(_dev(wl.to_nhwc(x)), packed, wg.NHWC, out=out)
    assert np.array_equal(wl.from_nhwc(out.cpu().numpy()), oracle.direct_conv2d(x, g))


@pytest.mark.parametrize("values", [(-128, -128), (127, -128), (-128, 127), (127, 127)])
def test_extreme_values_and_most_channels(values):
    """Every operand limb and the in-lane re-assembly at their limits; with C = 896 the intermediate sums wrap modulo
    2^32 and the result is still exact."""
    xv, gv = values
    for C in (64, wg.MAX_CHANNELS):
        x = np.full((1, C, 12, 8), xv, np.int8)
        g = np.full((10, C, 3, 3), gv, np.int8)
        g[1::2] = -gv if gv != -128 else 127
        packed = wg.winograd_filter_transform(_dev(wl.to_krsc(g)), wg.NHWC, wg.LOSSLESS)
        y = wg.winograd_conv2d_int8(_dev(wl.to_nhwc(x)), packed, wg.NHWC)
        assert np.array_equal(wl.from_nhwc(y.cpu().numpy()), oracle.direct_conv2d(x, g)), C


@pytest.mark.parametrize("offset", [0, 4, 8])
def test_input_alignment_selects_equivalent_load_paths(offset):
    N, C, K, H, W = 2, 80, 40, 11, 13
    x, g = wl.make_custom(N, C, K, H, W, seed=92)
    xs = wl.to_nhwc(x)
    buf = torch.zeros(xs.size + 16, dtype=torch.int8, device="cuda")
    xd = buf[offset:offset + xs.size].view(N, H, W, C)
    xd.copy_(torch.from_numpy(xs))
    assert xd.data_ptr() % 16 == offset
    packed = wg.winograd_filter_transform(_dev(wl.to_krsc(g)), wg.NHWC, wg.LOSSLESS)
    y = wg.winograd_conv2d_int8(xd, packed, wg.NHWC)
    assert np.array_equal(wl.from_nhwc(y.cpu().numpy()), oracle.direct_conv2d(x, g))


def test_output_canaries_and_unaligned_output():
    """Ragged H, W and an output pointer that is only 4-byte aligned: stores are clipped, guards stay intact."""
    N, C, K, H, W = 1, 16, 8, 7, 5
    x, g = wl.make_custom(N, C, K, H, W, seed=93)
    packed = wg.winograd_filter_transform(_dev(wl.to_krsc(g)), wg.NHWC, wg.LOSSLESS)
    n = N * H * W * K
    for lead in (64, 65):
        buf = torch.full((lead + n + 64,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
        out = buf[lead:lead + n].view(N, H, W, K)
        wg.winograd_conv2d_int8(_dev(wl.to_nhwc(x)), packed, wg.NHWC, out=out)
        assert np.array_equal(wl.from_nhwc(out.cpu().numpy()), oracle.direct_conv2d(x, g))
        assert (buf[:lead] == 0x5A5A5A5A).all() and (buf[-64:] == 0x5A5A5A5A).all()


@pytest.mark.parametrize("shape", [(2, 16, 32, 8, 12), (2, 20, 36, 10, 6), (1, 64, 7, 4, 4), (3, 32, 64, 18, 22), (1, 132, 68, 8, 8),
                                   (2, 16, 128, 40, 36), (1, 16, 6, 7, 9)])
def test_int8_epilogue_equals_oracle_conv_then_requantisation(shape):
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, seed=94)
    want32 = oracle.direct_conv2d(x, g)
    top = max(1, int(np.abs(want32).max()))
    packed = wg.winograd_filter_transform(_dev(wl.to_krsc(g)), wg.NHWC, wg.LOSSLESS)
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


def test_quoted_layer_both_forms_agree_with_the_oracle():
    """The 56x56x64 layer at its own batch: the limb-pair form (what the library picks there), the other form, and the
    oracle give the same bits."""
    x, g = wl.make_case("cfg2")
    xd, gd = _dev(wl.to_nhwc(x)), _dev(wl.to_krsc(g))
    packed = wg.winograd_filter_transform(gd, wg.NHWC, wg.LOSSLESS)
    y_pair = wg.winograd_conv2d_int8(xd, packed, wg.NHWC)
    wg.lossless_variant(2)
    y_other = wg.winograd_conv2d_int8(xd, packed, wg.NHWC)
    wg.lossless_variant(0)
    y_auto = wg.winograd_conv2d_int8(xd, packed, wg.NHWC)
    assert torch.equal(y_pair, y_other) and torch.equal(y_pair, y_auto)
    assert np.array_equal(wl.from_nhwc(y_pair.cpu().numpy()), oracle.direct_conv2d(x, g))
