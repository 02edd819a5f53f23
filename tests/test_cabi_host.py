"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function the header
declares, sizes are consistent, and every validation error path returns its code before any launch."""
import ctypes
import os
import re

import pytest

import paper_1901_01965_amd as wg
from paper_1901_01965_amd import binding, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "winograd_c.h")

OK, EINVAL, EUNSUPPORTED, ESMALLBUF = 0, -1, -2, -3


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_1901_01965_amd import build
        build.build()
    return wg.load_library()


def _declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(winograd_\w+|direct_conv2d_int8|requant_relu_pool_int8)\s*\(", text)))


def test_every_declared_function_is_exported(lib):
    names = _declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTED_SYMBOLS) == names


def test_status_strings(lib):
    for code in range(-6, 1):
        assert wg.binding.status_string(code)
    assert "blob" in wg.binding.status_string(-4)


def test_size_queries(lib):
    assert wg.packed_filter_bytes(0, 4, 0) == 0 and lib.winograd_packed_filter_bytes(4, 4, 7) == 0
    assert wg.packed_filter_bytes(4, 897, 0) == 0            # beyond WG_MAX_CHANNELS
    lossless, scaled = wg.packed_filter_bytes(64, 64, wg.LOSSLESS), wg.packed_filter_bytes(64, 64, wg.SCALED)
    assert lossless > 138 * 64 * 64 and scaled > 46 * 64 * 64 and lossless > scaled
    assert lossless % 256 == 0
    # padding: K up to 64, C up to 64
    assert wg.packed_filter_bytes(1, 5, 0) == wg.packed_filter_bytes(64, 64, 0)
    # up to four input channels: the blob also carries the 36 values of each filter as int16 x 4 channel slots
    assert wg.packed_filter_bytes(1, 1, 0) == wg.packed_filter_bytes(64, 4, 0) == wg.packed_filter_bytes(64, 64, 0) + 64 * 36 * 4 * 2
    assert wg.workspace_bytes(0, 1, 1, 1, 1, 0) == 0
    c = wl.CASES["cfg2"]
    ws = wg.workspace_bytes(c.N, c.C, c.H, c.W, c.K, wg.LOSSLESS)
    assert ws >= 138 * c.tiles * c.C + 36 * 4 * c.tiles * c.K
    assert lib.winograd_num_activation_planes(0) == 138 and lib.winograd_num_activation_planes(1) == 72
    assert lib.winograd_num_filter_planes(0) == 138 and lib.winograd_num_filter_planes(1) == 46
    assert lib.winograd_num_filter_planes(5) == 0


def test_path_query(lib):
    assert wg.conv2d_path(8, 64, 56, 56, 64, wg.LOSSLESS) == wg.FUSED
    assert wg.conv2d_path(64, 512, 7, 7, 512, wg.SCALED) == wg.FUSED
    assert lib.winograd_debug_force_path(wg.STAGED) == OK
    assert wg.conv2d_path(8, 64, 56, 56, 64, wg.LOSSLESS) == wg.STAGED
    assert lib.winograd_debug_force_path(wg.AUTO) == OK
    assert lib.winograd_conv2d_path(8, 64, 56, 56, 64, 9) == EINVAL
    assert lib.winograd_debug_force_path(3) == EINVAL
    assert lib.winograd_debug_force_path(0) == OK


def test_validation_errors_return_before_any_launch(lib):
    """Fake but well-aligned addresses: every call must be rejected on the host (nothing dereferences them)."""
    p = ctypes.c_void_p
    good, good2, good3 = p(0x10000), p(0x20000), p(0x30000)
    odd = p(0x10001)
    big = 1 << 40
    ft = lib.winograd_filter_transform
    assert ft(None, 4, 4, 0, 0, good, big, None) == EINVAL
    assert ft(good, 4, 4, 0, 0, None, big, None) == EINVAL
    assert ft(good, 0, 4, 0, 0, good2, big, None) == EINVAL
    assert ft(good, 4, -1, 0, 0, good2, big, None) == EINVAL
    assert ft(good, 4, 4, 2, 0, good2, big, None) == EINVAL          # unknown layout
    assert ft(good, 4, 4, 0, 2, good2, big, None) == EINVAL          # unknown mode
    assert ft(good, 4, 897, 0, 0, good2, big, None) == EUNSUPPORTED  # int32 exactness bound
    assert ft(odd, 4, 4, 0, 0, good2, big, None) == EINVAL           # misaligned filters
    assert ft(good, 4, 4, 0, 0, p(0x20010), big, None) == EINVAL     # misaligned blob
    assert ft(good, 4, 4, 0, 0, good2, 100, None) == ESMALLBUF

    conv = lib.winograd_conv2d_int8
    args = dict(N=1, C=4, H=8, W=8, K=4)
    ws_bytes = wg.workspace_bytes(1, 4, 8, 8, 4, 0)

    def call(x=good, blob=good2, y=good3, N=1, C=4, H=8, W=8, K=4, layout=0, mode=0, ws=p(0x40000), wsb=ws_bytes):
        return conv(x, blob, y, N, C, H, W, K, layout, mode, ws, wsb, None)

    assert call(x=None) == EINVAL and call(blob=None) == EINVAL and call(y=None) == EINVAL and call(ws=None) == EINVAL
    assert call(N=0) == EINVAL and call(H=-3) == EINVAL and call(K=0) == EINVAL
    assert call(layout=5) == EINVAL and call(mode=-1) == EINVAL
    assert call(C=1000) == EUNSUPPORTED
    assert call(N=1 << 20, H=1 << 10, W=1 << 10) == EUNSUPPORTED      # beyond 32-bit indexing
    assert call(wsb=ws_bytes - 1) == ESMALLBUF
    assert call(x=odd) == EINVAL and call(ws=p(0x40010)) == EINVAL

    direct = lib.direct_conv2d_int8
    assert direct(None, good, good2, 1, 4, 8, 8, 4, 0, None) == EINVAL
    assert direct(good, good2, good3, 1, 4, 8, 8, 4, 3, None) == EINVAL
    assert direct(good, good2, good3, 1, 900, 8, 8, 4, 0, None) == EUNSUPPORTED

    rq = lib.requant_relu_pool_int8
    assert rq(None, good, 1, 4, 8, 8, 0, 3, 1, 0, None) == EINVAL
    assert rq(good, good2, 1, 4, 8, 8, 0, 32, 1, 0, None) == EINVAL   # shift out of range
    assert rq(good, good2, 1, 4, 7, 8, 0, 3, 1, 1, None) == EUNSUPPORTED   # odd H with pooling

    cq = lib.winograd_conv2d_int8_requant
    assert cq(good, good2, None, 1, 4, 8, 8, 4, 0, 0, 3, 1, 0, None) == EINVAL
    assert cq(good, good2, good3, 1, 4, 8, 8, 4, 0, 0, -1, 1, 0, None) == EINVAL     # shift out of range
    assert cq(good, good2, good3, 1, 4, 8, 8, 4, 0, 0, 32, 1, 0, None) == EINVAL
    assert cq(good, good2, good3, 1, 4, 8, 8, 4, 0, 2, 3, 1, 0, None) == EINVAL      # unknown mode
    assert cq(good, good2, odd, 1, 4, 8, 8, 4, 0, 0, 3, 1, 0, None) == EINVAL        # misaligned output
    assert cq(good, good2, good3, 1, 4, 8, 7, 4, 0, 0, 3, 1, 1, None) == EUNSUPPORTED   # odd W with pooling
    assert cq(good, good2, good3, 1, 1000, 8, 8, 4, 0, 0, 3, 1, 0, None) == EUNSUPPORTED

    # rational F(2x2,3x3) entry points
    assert lib.winograd_f2x2_packed_filter_bytes(0, 4, 0) == 0 and lib.winograd_f2x2_packed_filter_bytes(4, 4, 5) == 0
    f2_bytes = lib.winograd_f2x2_packed_filter_bytes(4, 4, 0)
    assert f2_bytes > 32 * 64 * 64 and f2_bytes % 256 == 0
    assert lib.winograd_f2x2_packed_filter_bytes(4, 4, 1) < f2_bytes          # one operand plane per entry instead of two
    f2t = lib.winograd_f2x2_filter_transform
    assert f2t(None, 4, 4, 0, 0, good2, f2_bytes, None) == EINVAL
    assert f2t(good, 4, 4, 0, 0, good2, f2_bytes - 1, None) == ESMALLBUF
    assert f2t(good, 4, 1000, 0, 0, good2, big, None) == EUNSUPPORTED
    assert f2t(good, 4, 4, 0, 0, p(0x20010), big, None) == EINVAL             # misaligned blob
    f2c = lib.winograd_f2x2_conv2d_int8
    assert f2c(good, good2, None, 1, 4, 8, 8, 4, 0, 0, None) == EINVAL
    assert f2c(good, good2, good3, 1, 4, 8, 8, 4, 7, 0, None) == EINVAL       # unknown layout
    assert f2c(good, good2, good3, 0, 4, 8, 8, 4, 0, 0, None) == EINVAL
    assert f2c(odd, good2, good3, 1, 4, 8, 8, 4, 0, 0, None) == EINVAL
    assert f2c(good, good2, good3, 1, 1000, 8, 8, 4, 0, 0, None) == EUNSUPPORTED
    assert lib.winograd_f2x2_debug_filter_operands(good2, 4, 4, 0, None, good3, None) == EINVAL
    f2tu, f2cu = lib.winograd_f2x2_filter_transform_u8, lib.winograd_f2x2_conv2d_u8
    assert f2tu(good, 256, 4, 4, 0, 0, good2, f2_bytes, None) == EINVAL      # zero point beyond a byte
    assert f2tu(good, -1, 4, 4, 0, 0, good2, f2_bytes, None) == EINVAL
    assert f2tu(None, 3, 4, 4, 0, 0, good2, f2_bytes, None) == EINVAL
    assert f2cu(good, 300, good2, good3, 1, 4, 8, 8, 4, 0, 0, None) == EINVAL
    assert f2cu(good, 3, good2, None, 1, 4, 8, 8, 4, 0, 0, None) == EINVAL
    f2q = lib.winograd_f2x2_conv2d_int8_requant
    assert f2q(good, good2, None, 1, 4, 8, 8, 4, 0, 0, 3, 1, 0, None) == EINVAL
    assert f2q(good, good2, good3, 1, 4, 8, 8, 4, 0, 0, 32, 1, 0, None) == EINVAL        # shift out of range
    assert f2q(good, good2, good3, 1, 4, 8, 8, 4, 0, 2, 3, 1, 0, None) == EINVAL         # unknown mode
    assert f2q(good, good2, good3, 1, 4, 8, 7, 4, 0, 0, 3, 1, 1, None) == EUNSUPPORTED   # odd W with pooling
    f2a = lib.winograd_f2x2_conv2d_int8_act_scaled
    assert f2a(good, good2, None, 1, 4, 8, 8, 4, 0, None, None) == EINVAL
    assert f2a(good, None, good3, 1, 4, 8, 8, 4, 0, None, None) == EINVAL
    assert f2a(good, good2, good3, 1, 4, 8, 8, 4, 9, None, None) == EINVAL       # unknown layout
    assert f2a(good, good2, good3, 1, 4, 8, 8, 4, 0, odd, None) == EINVAL        # misaligned table export
    assert f2a(good, good2, good3, 1, 1000, 8, 8, 4, 0, None, None) == EUNSUPPORTED

    st = lib.winograd_conv2d_int8_enqueue_stage
    assert st(good, good2, good3, 1, 4, 8, 8, 4, 0, 0, p(0x40000), ws_bytes, None, 0, 0) == EINVAL    # iters < 1
    assert st(good, good2, good3, 1, 4, 8, 8, 4, 0, 0, p(0x40000), ws_bytes, None, 4, 1) == EINVAL    # unknown stage
    assert st(good, good2, good3, 1, 4, 8, 8, 4, 0, 0, None, ws_bytes, None, 0, 1) == EINVAL          # no workspace
    assert st(good, good2, good3, 1, 4, 8, 8, 4, 0, 0, p(0x40000), ws_bytes - 1, None, 0, 1) == ESMALLBUF
    assert lib.winograd_packed_filter_check(None, 4, 4, 0, None) == EINVAL
    assert lib.winograd_debug_input_operands(None, good, 1, 4, 8, 8, 0, 0, good2, big, None) == EINVAL
    assert lib.winograd_debug_filter_operands(good2, 4, 4, 3, good, good3, None) == EINVAL
    assert lib.winograd_debug_contraction(good, good2, good3, 1, 4, 8, 8, 4, 0, 0, None, big, None) == EINVAL


def test_binding_refuses_cpu_tensors(lib):
    import torch
    x = torch.zeros((1, 4, 8, 8), dtype=torch.int8)
    with pytest.raises(TypeError):
        wg.direct_conv2d_int8(x, torch.zeros((4, 4, 3, 3), dtype=torch.int8))


def test_vgg_shift_constants_match_the_generated_fixture():
    with open(os.path.join(ROOT, "tests", "golden", "vgg16_shifts.txt")) as f:
        line = [l for l in f if not l.startswith("#")][0]
    assert [int(t) for t in line.split()] == wl.VGG16_SHIFTS


def test_tile_decode_by_multiply_and_shift_matches_division(lib):
    """The kernels split a tile index with precomputed multiply-and-shift constants; compare with divmod
    over awkward tile grids, at the ends of every row and image."""
    out = (ctypes.c_int * 3)()
    shapes = [(1, 1, 1), (3, 4, 4), (5, 9, 7), (2, 56, 56), (16, 224, 224), (7, 13, 1021), (4000, 29, 31),
              (1, 4093, 4099), (65536, 8, 8)]
    for N, H, W in shapes:
        TH, TW = (H + 3) // 4, (W + 3) // 4
        T = N * TH * TW
        picks = {0, T - 1, T // 2, TW - 1, TW, TH * TW - 1, TH * TW, T - TW, max(0, T - TH * TW - 1)}
        picks |= {(i * 2654435761) % T for i in range(200)}
        for t in sorted(x for x in picks if 0 <= x < T):
            assert lib.winograd_debug_tile_decode(N, 4, H, W, 4, t, out) == 0
            n, rem = divmod(t, TH * TW)
            ty, tx = divmod(rem, TW)
            assert (out[0], out[1], out[2]) == (n, ty, tx), (N, H, W, t)
    assert lib.winograd_debug_tile_decode(1, 4, 8, 8, 4, 4, out) == EINVAL      # only 4 tiles
