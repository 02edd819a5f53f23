"""The entry points are enqueue-only (no allocation, no synchronisation): they can be recorded into a HIP graph, as
bench.py does.  Every replay must reproduce the eager result, with eager work of the program between the replays."""
import numpy as np
import pytest
import torch

import oracle
import paper_1901_01965_amd as wg
from paper_1901_01965_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", [wg.LOSSLESS, wg.SCALED])
def test_graph_replays_equal_eager_results(mode):
    N, C, K, H, W = 2, 80, 72, 12, 10
    x, g = wl.make_custom(N, C, K, H, W, act="relu", wgt="gauss", seed=81)
    x2, _ = wl.make_custom(N, C, K, H, W, act="relu", wgt="gauss", seed=82)
    xd = torch.from_numpy(wl.to_nhwc(x)).cuda()
    gd = torch.from_numpy(wl.to_krsc(g)).cuda()
    packed = wg.winograd_filter_transform(gd, wg.NHWC, mode)
    packed2 = wg.f2x2_filter_transform(gd, wg.NHWC, mode)
    ws = wg.make_workspace(N, C, H, W, K, mode)
    y = torch.empty((N, H, W, K), dtype=torch.int32, device="cuda")
    q = torch.empty((N, H // 2, W // 2, K), dtype=torch.int8, device="cuda")
    y2 = torch.empty_like(y)
    y3 = torch.empty_like(y)
    yd = torch.empty_like(y)

    def work():
        wg.winograd_conv2d_int8(xd, packed, wg.NHWC, out=y, workspace=ws)
        wg.winograd_conv2d_int8_requant(xd, packed, 10, True, True, wg.NHWC, out=q)
        wg.f2x2_conv2d_int8(xd, packed2, wg.NHWC, out=y2)
        if mode == wg.SCALED:
            wg.f2x2_conv2d_int8_act_scaled(xd, packed2, wg.NHWC, out=y3)
        wg.direct_conv2d_int8(xd, gd, wg.NHWC, out=yd)

    work()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        work()
    inputs = [x, x2, x]
    for xin in inputs:
        xd.copy_(torch.from_numpy(wl.to_nhwc(xin)).cuda())       # eager work between the replays
        for t in (y, y2, y3, yd):
            t.fill_(-7)
        q.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        if mode == wg.LOSSLESS:
            want = oracle.direct_conv2d(xin, g)
            want2 = want
        else:
            want = oracle.winograd_conv2d(xin, g, oracle.SCALED, 127)[0]
            want2 = oracle.f2_conv2d(xin, g, oracle.SCALED, 127)[0]
        assert np.array_equal(wl.from_nhwc(y.cpu().numpy()), want)
        assert np.array_equal(wl.from_nhwc(q.cpu().numpy()), oracle.requant_relu_pool(want, 10, True, True))
        assert np.array_equal(wl.from_nhwc(y2.cpu().numpy()), want2)
        if mode == wg.SCALED:
            assert np.array_equal(wl.from_nhwc(y3.cpu().numpy()), oracle.f2_conv2d(xin, g, oracle.BOTH_SCALED, 127)[0])
        assert np.array_equal(wl.from_nhwc(yd.cpu().numpy()), oracle.direct_conv2d(xin, g))
