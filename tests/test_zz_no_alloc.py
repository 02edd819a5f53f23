"""The entry point that allocates nothing (winograd_conv2d_int8_static_workspace: the staged pipeline through the
scratch buffer inside the library) against winograd_conv2d_int8 on its staged path with a caller's workspace,
through the C ABI, bit for bit; two calls in a row, the second with a smaller input."""
import ctypes
import gc

import numpy as np
import pytest
import torch

import oracle
import paper_1901_01965_amd as wg
from paper_1901_01965_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _both(lib, x, g, mode):
    N, C, H, W = x.shape
    K = g.shape[0]
    xd = torch.from_numpy(wl.to_nhwc(x)).cuda()
    packed = wg.winograd_filter_transform(torch.from_numpy(wl.to_krsc(g)).cuda(), wg.NHWC, mode)
    ws = wg.make_workspace(N, C, H, W, K, mode)
    want = torch.full((N, H, W, K), 123456, dtype=torch.int32, device="cuda")
    got = torch.full((N, H, W, K), 654321, dtype=torch.int32, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    wg.force_path(wg.STAGED)
    try:
        assert lib.winograd_conv2d_int8(p(xd), p(packed.blob), p(want), N, C, H, W, K, wg.NHWC, mode, p(ws), ws.numel(),
                                        stream) == 0
    finally:
        wg.force_path(wg.AUTO)
    torch.cuda.synchronize()
    # Free device memory as the runtime reports it must not drop across the call (nothing else runs meanwhile; torch's
    # own allocator is not involved in a ctypes call, and a collection here keeps stray frees out of the window).  The
    # process's first call is left out: that is when the runtime places the library's device image, the 64 MiB array
    # included, on the GPU.
    gc.collect()
    before = torch.cuda.mem_get_info()[0]
    assert lib.winograd_conv2d_int8_static_workspace(p(xd), p(packed.blob), p(got), N, C, H, W, K, wg.NHWC, mode,
                                                     stream) == 0
    torch.cuda.synchronize()
    if _both.calls > 0:
        assert torch.cuda.mem_get_info()[0] >= before
    _both.calls += 1
    return got.cpu().numpy(), want.cpu().numpy()


_both.calls = 0


@pytest.mark.parametrize("mode", [wg.LOSSLESS, wg.SCALED])
def test_static_workspace_entry_point_equals_the_workspace_one_twice_in_a_row(mode):
    lib = wg.load_library()
    big = wl.make_custom(3, 70, 40, 30, 26, act="uniform", wgt="uniform", seed=81)    # ragged tiles, two channel blocks
    small = wl.make_custom(1, 24, 33, 9, 7, act="uniform", wgt="uniform", seed=82)    # fewer tiles, channels and filters
    for x, g in (big, small):
        got, want = _both(lib, x, g, mode)
        assert np.array_equal(got, want)
        ref = oracle.direct_conv2d(x, g) if mode == wg.LOSSLESS else oracle.winograd_conv2d(x, g, oracle.SCALED)[0]
        assert np.array_equal(wl.from_nhwc(got), ref)


def test_static_workspace_entry_point_rejects_what_does_not_fit():
    lib = wg.load_library()
    limit = wg.static_workspace_limit()
    assert limit == 64 << 20
    N, C, H, W, K = 8, 64, 56, 56, 64
    assert wg.workspace_bytes(N, C, H, W, K, wg.LOSSLESS) <= limit < wg.workspace_bytes(4 * N, C, H, W, K, wg.LOSSLESS)
    x = torch.zeros((4 * N, H, W, C), dtype=torch.int8, device="cuda")
    g = torch.zeros((K, 3, 3, C), dtype=torch.int8, device="cuda")
    packed = wg.winograd_filter_transform(g, wg.NHWC, wg.LOSSLESS)
    with pytest.raises(wg.WinogradError) as err:
        wg.winograd_conv2d_int8_static_workspace(x, packed, wg.NHWC)
    assert err.value.status == -3
    # the quoted layer fits: the whole buffer is in use, and the result is the direct convolution
    xs, gs = wl.make_case("cfg2")
    xd, gd = torch.from_numpy(wl.to_nhwc(xs)).cuda(), torch.from_numpy(wl.to_krsc(gs)).cuda()
    y = wg.winograd_conv2d_int8_static_workspace(xd, wg.winograd_filter_transform(gd, wg.NHWC, wg.LOSSLESS), wg.NHWC)
    assert torch.equal(y, wg.direct_conv2d_int8(xd, gd, wg.NHWC))
