"""GPU parity at the full sizes of the five benchmark configurations, through the C ABI, in the launch
configuration bench.py times (library's own path choice), bit for bit against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_1901_01965_amd as wg
from paper_1901_01965_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _run(x, g, layout, mode, path=wg.AUTO):
    wg.force_path(path)
    try:
        xd = torch.from_numpy(x if layout == wg.NCHW else wl.to_nhwc(x)).cuda()
        gd = torch.from_numpy(g if layout == wg.NCHW else wl.to_krsc(g)).cuda()
        packed = wg.winograd_filter_transform(gd, layout, mode)
        packed.check()
        y = wg.winograd_conv2d_int8(xd, packed, layout).cpu().numpy()
    finally:
        wg.force_path(wg.AUTO)
    return y if layout == wg.NCHW else wl.from_nhwc(y)


def _report(name, got_scaled, direct):
    err = np.abs(got_scaled.astype(np.int64) - direct.astype(np.int64))
    print("\n%s scaled-mode error vs direct: max %d, mean %.3f (mean |y| %.1f)"
          % (name, err.max(), err.mean(), np.abs(direct).mean()))


@pytest.mark.parametrize("layout", [wg.NHWC, wg.NCHW])
def test_cfg1_lossless(layout):
    x, g = wl.make_case("cfg1")
    assert np.array_equal(_run(x, g, layout, wg.LOSSLESS), oracle.direct_conv2d(x, g))


@pytest.mark.parametrize("path", [wg.AUTO, wg.STAGED])
@pytest.mark.parametrize("layout", [wg.NHWC, wg.NCHW])
def test_cfg2_lossless(layout, path):
    x, g = wl.make_case("cfg2")
    assert np.array_equal(_run(x, g, layout, wg.LOSSLESS, path), oracle.direct_conv2d(x, g))


@pytest.mark.parametrize("path", [wg.AUTO, wg.STAGED])
def test_cfg3_lossless_and_scaled(path):
    x, g = wl.make_case("cfg3")
    direct = oracle.direct_conv2d(x, g)
    assert np.array_equal(_run(x, g, wg.NHWC, wg.LOSSLESS, path), direct)
    want, flags = oracle.winograd_conv2d(x, g, oracle.SCALED, 127)
    assert (flags & 5) == 0
    got = _run(x, g, wg.NHWC, wg.SCALED, path)
    assert np.array_equal(got, want)
    _report("cfg3", got, direct)


@pytest.mark.parametrize("name", ["cfg4a", "cfg4b"])
def test_cfg4_scaled(name):
    x, g = wl.make_case(name)
    want, flags = oracle.winograd_conv2d(x, g, oracle.SCALED, 127)
    assert (flags & 5) == 0
    try:
        for path in (wg.STAGED, wg.FUSED):   # both implementations at full size
            wg.force_path(path)
            got = _run(x, g, wg.NHWC, wg.SCALED)
            assert np.array_equal(got, want), path
    finally:
        wg.force_path(wg.AUTO)
    _report(name, got, oracle.direct_conv2d(x, g))
    # the same layers in lossless mode, and in the other layout
    assert np.array_equal(_run(x, g, wg.NCHW, wg.LOSSLESS), oracle.direct_conv2d(x, g))


def _vgg_stack_gpu(x, gs, mode, layers, keep=slice(None)):
    """Runs `layers` of the stack on the GPU (channels-last); returns, for the images `keep`, every layer's int8
    input, int32 output and int8 requantised output as NCHW numpy arrays."""
    act = torch.from_numpy(wl.to_nhwc(x)).cuda()
    outs = []
    for i in layers:
        cin, cout, hw, pool = wl.VGG16_LAYERS[i]
        gd = torch.from_numpy(wl.to_krsc(gs[i])).cuda()
        packed = wg.winograd_filter_transform(gd, wg.NHWC, mode)
        y = wg.winograd_conv2d_int8(act, packed, wg.NHWC)
        nxt = wg.requant_relu_pool_int8(y, wl.VGG16_SHIFTS[i], True, pool, wg.NHWC)
        # the same layer with the requantisation inside the convolution kernel; nxt itself is checked
        # against the oracle by the callers
        one_kernel = wg.winograd_conv2d_int8_requant(act, packed, wl.VGG16_SHIFTS[i], True, pool, wg.NHWC)
        assert torch.equal(one_kernel, nxt), "layer %d: int8 epilogue differs from the two-kernel result" % i
        outs.append(tuple(wl.from_nhwc(t[keep].cpu().numpy()) for t in (act, y, nxt)))
        act = nxt
        del y
    return outs


@pytest.mark.parametrize("mode", [wg.LOSSLESS, wg.SCALED])
def test_cfg5_vgg16_stack_one_image(mode):
    """All 13 layers with requantisation, ReLU and pooling.  Each layer is checked on its own: the oracle
    gets the GPU's (already verified) int8 input of that layer, so one layer's check does not depend on
    the others and the scaled mode's small errors do not compound in the comparison."""
    x, gs = wl.make_vgg16(batch=1)
    outs = _vgg_stack_gpu(x, gs, mode, range(13))
    layer_in = x
    for i, (gpu_in, y, nxt) in enumerate(outs):
        cin, cout, hw, pool = wl.VGG16_LAYERS[i]
        assert np.array_equal(gpu_in, layer_in)
        if mode == wg.LOSSLESS:
            want = oracle.direct_conv2d(layer_in, gs[i])
        else:
            want, flags = oracle.winograd_conv2d(layer_in, gs[i], oracle.SCALED, 127)
            assert (flags & 5) == 0
        assert np.array_equal(y, want), "layer %d" % i
        assert np.array_equal(nxt, oracle.requant_relu_pool(want, wl.VGG16_SHIFTS[i], True, pool)), "layer %d" % i
        assert (nxt != 0).mean() > 0.2 and nxt.max() > 32, "activations died out at layer %d" % i
        layer_in = nxt


@pytest.mark.parametrize("mode", [wg.LOSSLESS, wg.SCALED])
def test_cfg5_vgg16_stack_full_batch(mode):
    """All 13 layers at the stack's own batch of 16, where the library picks other kernel variants than at
    batch 1 (streaming, role-specialised, 64-filter workgroups).  The oracle checks the last image of every
    layer, whose tiles sit at the far end of every buffer: it is given the GPU's int8 input of that layer (the
    scheme of the one-image test), so a layer's check does not depend on the layers before it."""
    x, gs = wl.make_vgg16(batch=wl.VGG16_BATCH)
    outs = _vgg_stack_gpu(x, gs, mode, range(13), keep=slice(wl.VGG16_BATCH - 1, wl.VGG16_BATCH))
    assert np.array_equal(outs[0][0], x[-1:])
    for i, (layer_in, y, nxt) in enumerate(outs):
        cin, cout, hw, pool = wl.VGG16_LAYERS[i]
        if mode == wg.LOSSLESS:
            want = oracle.direct_conv2d(layer_in, gs[i])
        else:
            want, flags = oracle.winograd_conv2d(layer_in, gs[i], oracle.SCALED, 127)
            assert (flags & 5) == 0
        assert np.array_equal(y, want), "layer %d" % i
        assert np.array_equal(nxt, oracle.requant_relu_pool(want, wl.VGG16_SHIFTS[i], True, pool)), "layer %d" % i
        if i + 1 < 13:
            assert np.array_equal(outs[i + 1][0], nxt), "layer %d: the next layer did not get this output" % i
        print("layer %d ok" % i, flush=True)
