"""GPU parity: every stage and the whole path, through the C ABI, bit for bit against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_1901_01965_amd as wg
from paper_1901_01965_amd import workloads as wl

pytestmark = pytest.mark.gpu

R = (0, 1, 2, 5)
# the library's order of the 26 free entries
ENTRIES = [(r, c) for r in R for c in R] + [(r, 3) for r in R] + [(3, c) for c in R] + [(3, 3), (3, 4)]


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _x(x, layout):
    return _dev(x if layout == wg.NCHW else wl.to_nhwc(x))


def _g(g, layout):
    return _dev(g if layout == wg.NCHW else wl.to_krsc(g))


def _y(y, layout):
    y = y.cpu().numpy()
    return y if layout == wg.NCHW else wl.from_nhwc(y)


def _values_from_oracle(X):
    """Oracle tiles [A, B, 6, 6, 2] -> the library's 46 'values' [46, A, B]: 16 real entries, then
    (Re, Im, Re+Im) of each complex entry."""
    vals = [X[:, :, r, c, 0] for (r, c) in ENTRIES[:16]]
    for (r, c) in ENTRIES[16:]:
        vals += [X[:, :, r, c, 0], X[:, :, r, c, 1], X[:, :, r, c, 0] + X[:, :, r, c, 1]]
    return np.stack(vals)


def _check_lossless_planes(planes, X):
    """planes int8 [138, A, B]: 3v = v >> 6, 3v+1 = v & 63, 3v+2 = their sum."""
    vals = _values_from_oracle(X)
    planes = planes.astype(np.int64)
    assert np.array_equal(planes[0::3], vals >> 6)
    assert np.array_equal(planes[1::3], vals & 63)
    assert np.array_equal(planes[2::3], (vals >> 6) + (vals & 63))
    assert np.array_equal(64 * planes[0::3] + planes[1::3], vals)


SHAPES = [  # N, C, K, H, W
    (1, 4, 4, 4, 4), (1, 3, 5, 7, 9), (2, 16, 16, 16, 16), (1, 70, 33, 10, 6), (3, 8, 100, 5, 13),
    (1, 1, 1, 1, 1), (1, 130, 65, 8, 8),
]
LAYOUTS = [wg.NHWC, wg.NCHW]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("shape", SHAPES)
def test_input_transform_lossless_planes(shape, layout):
    N, C, K, H, W = shape
    x, _ = wl.make_custom(N, C, K, H, W, seed=31)
    planes = wg.debug_input_operands(_x(x, layout), layout, wg.LOSSLESS).cpu().numpy()
    _check_lossless_planes(planes, oracle.input_transform(x))


@pytest.mark.parametrize("layout", LAYOUTS)
def test_input_transform_scaled_planes(layout):
    x, _ = wl.make_custom(2, 20, 3, 9, 11, seed=32)
    planes = wg.debug_input_operands(_x(x, layout), layout, wg.SCALED).cpu().numpy().astype(np.int64)
    D = oracle.input_transform(x)
    want = []
    for (r, c) in ENTRIES[:16]:
        want += [D[:, :, r, c, 0] >> 6, D[:, :, r, c, 0] & 63]
    for (r, c) in ENTRIES[16:]:
        want += [D[:, :, r, c, 0] >> 6, D[:, :, r, c, 0] & 63, D[:, :, r, c, 1] >> 6, D[:, :, r, c, 1] & 63]
    assert np.array_equal(planes, np.stack(want))


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("kc", [(4, 4), (5, 3), (64, 64), (33, 70), (130, 65)])
def test_filter_transform_lossless_planes(kc, layout):
    K, C = kc
    _, g = wl.make_custom(1, C, K, 4, 4, seed=33)
    packed = wg.winograd_filter_transform(_g(g, layout), layout, wg.LOSSLESS)
    packed.check()
    planes, table = wg.debug_filter_operands(packed)
    _check_lossless_planes(planes.cpu().numpy(), oracle.filter_transform(g))
    table = table.cpu().numpy()
    assert (table == np.array([0, 0, 1, 0])).all()


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("kc,wgt", [((4, 4), "uniform"), ((5, 3), "gauss"), ((64, 64), "gauss"), ((33, 70), "uniform")])
def test_filter_transform_scaled_planes_and_table(kc, wgt, layout):
    K, C = kc
    _, g = wl.make_custom(1, C, K, 4, 4, wgt=wgt, seed=34)
    packed = wg.winograd_filter_transform(_g(g, layout), layout, wg.SCALED)
    planes, table = wg.debug_filter_operands(packed)
    planes, table = planes.cpu().numpy().astype(np.int64), table.cpu().numpy()
    Ws, tab, _ = oracle.scale_filters(oracle.filter_transform(g), 127)
    want = [Ws[:, :, r, c, 0] for (r, c) in ENTRIES[:16]]
    for (r, c) in ENTRIES[16:]:
        want += [Ws[:, :, r, c, 0], Ws[:, :, r, c, 1], -Ws[:, :, r, c, 1]]
    assert np.array_equal(planes, np.stack(want))
    want_tab = np.stack([tab[:, r, c] for (r, c) in ENTRIES], axis=1)
    assert np.array_equal(table, want_tab)


def _accumulators_from_oracle(M):
    planes = [M[:, :, r, c, 0] for (r, c) in ENTRIES[:16]]
    for (r, c) in ENTRIES[16:]:
        planes += [M[:, :, r, c, 0], M[:, :, r, c, 1]]
    return np.stack(planes)


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("mode", [wg.LOSSLESS, wg.SCALED])
@pytest.mark.parametrize("shape", [(1, 4, 4, 4, 4), (2, 16, 16, 16, 16), (1, 70, 33, 10, 6), (1, 130, 65, 8, 8)])
def test_contraction_accumulators(shape, mode, layout):
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, wgt="gauss" if mode == wg.SCALED else "uniform", seed=35)
    packed = wg.winograd_filter_transform(_g(g, layout), layout, mode)
    got = wg.debug_contraction(_x(x, layout), packed, layout).cpu().numpy()
    D, Wt = oracle.input_transform(x), oracle.filter_transform(g)
    if mode == wg.SCALED:
        Ws, tab, _ = oracle.scale_filters(Wt, 127)
        M = oracle.inverse_scale(oracle.contract(D, Ws), tab)
    else:
        M = oracle.contract(D, Wt)
    want = _accumulators_from_oracle(M)
    assert np.array_equal(got.astype(np.int64), want)      # every accumulator fits int32 at these sizes


E2E_SHAPES = SHAPES + [(2, 64, 64, 12, 12), (1, 32, 48, 30, 18), (1, 200, 40, 9, 9)]
PATHS = [wg.STAGED, wg.FUSED]


@pytest.fixture
def path(request):
    """Pins winograd_conv2d_int8 to one implementation for the test, then restores the default."""
    wg.force_path(request.param)
    yield request.param
    wg.force_path(wg.AUTO)



@pytest.mark.parametrize("path", PATHS, indirect=True)
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("shape", E2E_SHAPES)
def test_lossless_conv_equals_oracle_direct(shape, layout, path):
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, seed=36)
    packed = wg.winograd_filter_transform(_g(g, layout), layout, wg.LOSSLESS)
    y = wg.winograd_conv2d_int8(_x(x, layout), packed, layout)
    assert np.array_equal(_y(y, layout), oracle.direct_conv2d(x, g))


@pytest.mark.parametrize("path", PATHS, indirect=True)
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("shape", E2E_SHAPES)
def test_scaled_conv_equals_oracle_scaled(shape, layout, path):
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, act="relu", wgt="gauss", seed=37)
    packed = wg.winograd_filter_transform(_g(g, layout), layout, wg.SCALED)
    y = wg.winograd_conv2d_int8(_x(x, layout), packed, layout)
    want, flags = oracle.winograd_conv2d(x, g, oracle.SCALED, 127)
    assert (flags & 5) == 0
    assert np.array_equal(_y(y, layout), want)


@pytest.mark.parametrize("mode", [wg.LOSSLESS, wg.SCALED])
@pytest.mark.parametrize("offset", [0, 4, 8])
def test_channels_last_input_alignment_selects_equivalent_load_paths(offset, mode):
    """Channels-last inputs with C % 16 == 0 are moved in 16-byte pieces only when the pointer is 16-byte
    aligned; a pointer that is only 4-byte aligned takes the 4-byte loads.  Same results either way."""
    N, C, K, H, W = 2, 80, 40, 11, 13
    x, g = wl.make_custom(N, C, K, H, W, act="relu", wgt="gauss", seed=41)
    xs = np.ascontiguousarray(wl.to_nhwc(x))
    buf = torch.zeros(xs.size + 16, dtype=torch.int8, device="cuda")
    xd = buf[offset:offset + xs.size].view(N, H, W, C)
    xd.copy_(torch.from_numpy(xs))
    assert xd.data_ptr() % 16 == offset
    packed = wg.winograd_filter_transform(_g(g, wg.NHWC), wg.NHWC, mode)
    y = wg.winograd_conv2d_int8(xd, packed, wg.NHWC)
    if mode == wg.LOSSLESS:
        want = oracle.direct_conv2d(x, g)
    else:
        want, flags = oracle.winograd_conv2d(x, g, oracle.SCALED, 127)
        assert (flags & 5) == 0
    assert np.array_equal(_y(y, wg.NHWC), want)


@pytest.mark.parametrize("mode", [wg.LOSSLESS, wg.SCALED])
def test_many_tiles_ragged_filters(mode):
    """More (tile block, 32-filter block) pairs than compute units: the fused kernel then covers 64 filters per
    workgroup (two passes over the entries).  K = 72 leaves the last pass of the last workgroup mostly padding;
    H = W = 131 leaves ragged tiles."""
    N, C, K, H, W = 1, 16, 72, 131, 131
    assert ((H + 3) // 4) * ((W + 3) // 4) // 16 * ((K + 63) // 64 * 2) > 256
    x, g = wl.make_custom(N, C, K, H, W, act="relu", wgt="gauss", seed=42)
    packed = wg.winograd_filter_transform(_g(g, wg.NHWC), wg.NHWC, mode)
    y = wg.winograd_conv2d_int8(_x(x, wg.NHWC), packed, wg.NHWC)
    if mode == wg.LOSSLESS:
        want = oracle.direct_conv2d(x, g)
    else:
        want, flags = oracle.winograd_conv2d(x, g, oracle.SCALED, 127)
        assert (flags & 5) == 0
    assert np.array_equal(_y(y, wg.NHWC), want)


@pytest.mark.parametrize("path", PATHS, indirect=True)
@pytest.mark.parametrize("layout", LAYOUTS)
def test_extreme_values_lossless(layout, path):
    """All-extreme int8 data drives every 12-bit operand and the limb recombination to their limits."""
    for xv, gv in ((-128, -128), (127, -128), (-128, 127)):
        x = np.full((1, 64, 8, 8), xv, np.int8)
        g = np.full((8, 64, 3, 3), gv, np.int8)
        packed = wg.winograd_filter_transform(_g(g, layout), layout, wg.LOSSLESS)
        y = wg.winograd_conv2d_int8(_x(x, layout), packed, layout)
        assert np.array_equal(_y(y, layout), oracle.direct_conv2d(x, g))


@pytest.mark.parametrize("mode", [wg.LOSSLESS, wg.SCALED])
@pytest.mark.parametrize("C", [1, 3, 4])
def test_extreme_values_narrow_input(C, mode):
    """All-extreme data through the vector-ALU kernel (C <= 4, channels-last): its 16-bit operands and the
    24-bit products summed over four channel slots are at their largest."""
    for xv, gv in ((-128, -128), (127, -128), (-128, 127), (127, 127)):
        x = np.full((1, C, 12, 8), xv, np.int8)
        g = np.full((66, C, 3, 3), gv, np.int8)
        g[1::2] = -gv if gv != -128 else 127
        packed = wg.winograd_filter_transform(_g(g, wg.NHWC), wg.NHWC, mode)
        y = wg.winograd_conv2d_int8(_x(x, wg.NHWC), packed, wg.NHWC)
        want = oracle.direct_conv2d(x, g) if mode == wg.LOSSLESS else oracle.winograd_conv2d(x, g, oracle.SCALED)[0]
        assert np.array_equal(_y(y, wg.NHWC), want), (xv, gv)


@pytest.mark.parametrize("path", PATHS, indirect=True)
def test_max_channels_lossless_wraparound_is_exact(path):
    """C = 896 with worst-case data: intermediate accumulators wrap modulo 2^32, the result is exact."""
    C = wg.MAX_CHANNELS
    x = np.full((1, C, 4, 4), -128, np.int8)
    g = np.full((2, C, 3, 3), -128, np.int8)
    g[1] = 127
    packed = wg.winograd_filter_transform(_g(g, wg.NHWC), wg.NHWC, wg.LOSSLESS)
    y = wg.winograd_conv2d_int8(_x(x, wg.NHWC), packed, wg.NHWC)
    assert np.array_equal(_y(y, wg.NHWC), oracle.direct_conv2d(x, g))


# plus shapes for the matrix-core direct kernel (channels-last, C % 16 == 0, K % 4 == 0): several
# channel blocks with a ragged last one, ragged patches, more than 64 filters
DIRECT_SHAPES = E2E_SHAPES + [(1, 144, 72, 9, 20), (2, 16, 132, 17, 33), (1, 64, 4, 8, 16)]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("shape", DIRECT_SHAPES)
def test_direct_conv_equals_oracle(shape, layout):
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, seed=38)
    y = wg.direct_conv2d_int8(_x(x, layout), _g(g, layout), layout)
    assert np.array_equal(_y(y, layout), oracle.direct_conv2d(x, g))


@pytest.mark.parametrize("layout", LAYOUTS)
def test_requant_relu_pool(layout):
    rng = np.random.default_rng(39)
    y = rng.integers(-40000, 40000, (2, 5, 6, 8)).astype(np.int32)
    for shift in (0, 3, 9):
        for relu in (True, False):
            for pool in (True, False):
                got = wg.requant_relu_pool_int8(_x(y, layout), shift, relu, pool, layout)
                assert np.array_equal(_y(got, layout), oracle.requant_relu_pool(y, shift, relu, pool))


REQUANT_SHAPES = [  # N, C, K, H, W: every load variant, both store paths, ragged tiles and filters, 64-filter groups
    (2, 16, 32, 8, 12), (1, 3, 5, 6, 10), (2, 20, 36, 10, 6), (1, 70, 33, 12, 8), (1, 64, 7, 4, 4),
    (3, 32, 64, 18, 22), (1, 130, 68, 8, 8), (5, 16, 128, 40, 36), (1, 1, 1, 2, 2),
]


@pytest.mark.parametrize("mode", [wg.LOSSLESS, wg.SCALED])
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("shape", REQUANT_SHAPES)
def test_conv_with_int8_epilogue_equals_oracle_conv_then_requantisation(shape, layout, mode):
    """The int8 store of the single-kernel path against the oracle's convolution followed by the oracle's
    requantisation, ReLU and pooling; the shift is chosen so that the outputs spread over the int8 range and some
    saturate."""
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, seed=58)
    want32 = oracle.direct_conv2d(x, g) if mode == wg.LOSSLESS else oracle.winograd_conv2d(x, g, oracle.SCALED)[0]
    top = max(1, int(np.abs(want32).max()))
    shifts = sorted({0, max(0, top.bit_length() - 8), max(0, top.bit_length() - 6)})
    packed = wg.winograd_filter_transform(_g(g, layout), layout, mode)
    xd = _x(x, layout)
    for shift in shifts:
        for relu in (True, False):
            for pool in (False, True):
                got = wg.winograd_conv2d_int8_requant(xd, packed, shift, relu, pool, layout)
                assert np.array_equal(_y(got, layout), oracle.requant_relu_pool(want32, shift, relu, pool)), (
                    shift, relu, pool)


def test_int8_epilogue_odd_sizes_without_pooling_and_fill():
    """Odd H and W (ragged tiles) without pooling; the output buffer is pre-filled so that an element the kernel
    skipped would show."""
    x, g = wl.make_custom(2, 24, 40, 7, 13, seed=59)
    want32 = oracle.direct_conv2d(x, g)
    for layout in LAYOUTS:
        packed = wg.winograd_filter_transform(_g(g, layout), layout, wg.LOSSLESS)
        shape = (2, 40, 7, 13) if layout == wg.NCHW else (2, 7, 13, 40)
        out = torch.full(shape, 77, dtype=torch.int8, device="cuda")
        wg.winograd_conv2d_int8_requant(_x(x, layout), packed, 9, False, False, layout, out=out)
        assert np.array_equal(_y(out, layout), oracle.requant_relu_pool(want32, 9, False, False))
        with pytest.raises(wg.WinogradError):
            wg.winograd_conv2d_int8_requant(_x(x, layout), packed, 9, True, True, layout)


NARROW_SHAPES = [  # N, C, K, H, W: at most four input channels, channels-last -> the vector-ALU kernel
    (2, 3, 70, 30, 22), (1, 1, 64, 16, 16), (3, 2, 5, 9, 7), (1, 4, 130, 20, 36), (1, 3, 64, 4, 4),
]


@pytest.mark.parametrize("mode", [wg.LOSSLESS, wg.SCALED])
@pytest.mark.parametrize("wgt", ["uniform", "gauss"])
@pytest.mark.parametrize("shape", NARROW_SHAPES)
def test_narrow_input_layers(shape, wgt, mode):
    """First-layer shapes (C <= 4, channels-last): int32 output and the int8 epilogue, more than one wave's 64 tiles,
    more than 64 filters, ragged tiles and filter counts; uniform weights make most locations need scaling."""
    N, C, K, H, W = shape
    x, g = wl.make_custom(N, C, K, H, W, wgt=wgt, seed=61)
    want = oracle.direct_conv2d(x, g) if mode == wg.LOSSLESS else oracle.winograd_conv2d(x, g, oracle.SCALED)[0]
    packed = wg.winograd_filter_transform(_g(g, wg.NHWC), wg.NHWC, mode)
    xd = _x(x, wg.NHWC)
    assert np.array_equal(_y(wg.winograd_conv2d_int8(xd, packed, wg.NHWC), wg.NHWC), want)
    shift = max(0, int(np.abs(want).max()).bit_length() - 7)
    for relu in (True, False):
        for pool in (False, True):
            if pool and (H % 2 or W % 2):
                continue
            got = wg.winograd_conv2d_int8_requant(xd, packed, shift, relu, pool, wg.NHWC)
            assert np.array_equal(_y(got, wg.NHWC), oracle.requant_relu_pool(want, shift, relu, pool)), (relu, pool)
    # the staged pipeline on the same blob gives the same int32 result
    wg.force_path(wg.STAGED)
    try:
        assert np.array_equal(_y(wg.winograd_conv2d_int8(xd, packed, wg.NHWC), wg.NHWC), want)
    finally:
        wg.force_path(wg.AUTO)


STREAM_CASES = [  # (N, C, K, H, W), workgroups per filter block: tile blocks per workgroup 1, several, uneven;
    # one to three channel blocks; ragged last tile block; filters beyond K in the last block
    ((1, 16, 32, 16, 16), 1), ((2, 16, 32, 20, 16), 3), ((3, 64, 40, 18, 22), 4), ((2, 80, 72, 14, 14), 2),
    ((1, 132, 36, 26, 10), 5), ((4, 32, 64, 8, 8), 7), ((1, 200, 32, 9, 7), 1),
]


@pytest.mark.parametrize("mode", [wg.LOSSLESS, wg.SCALED])
@pytest.mark.parametrize("case", STREAM_CASES)
def test_streaming_variant_of_the_single_kernel_path(case, mode):
    """The role-specialised streaming kernel (a workgroup walks over several tile blocks; transform waves one unit
    ahead of product waves and storing the previous tile block), forced through the test hook on small problems:
    int32 output and the int8 epilogue with and without pooling."""
    (N, C, K, H, W), slots = case
    x, g = wl.make_custom(N, C, K, H, W, act="relu", wgt="gauss", seed=63)
    want = oracle.direct_conv2d(x, g) if mode == wg.LOSSLESS else oracle.winograd_conv2d(x, g, oracle.SCALED)[0]
    packed = wg.winograd_filter_transform(_g(g, wg.NHWC), wg.NHWC, mode)
    xd = _x(x, wg.NHWC)
    shift = max(0, int(np.abs(want).max()).bit_length() - 7)
    wg.stream_workgroups(slots)
    try:
        out = torch.full((N, H, W, K), 1357911, dtype=torch.int32, device="cuda")
        wg.winograd_conv2d_int8(xd, packed, wg.NHWC, out=out)
        assert np.array_equal(_y(out, wg.NHWC), want)
        for pool in (False, True):
            if pool and (H % 2 or W % 2):
                continue
            got = wg.winograd_conv2d_int8_requant(xd, packed, shift, True, pool, wg.NHWC)
            assert np.array_equal(_y(got, wg.NHWC), oracle.requant_relu_pool(want, shift, True, pool)), pool
    finally:
        wg.stream_workgroups(0)


def test_streaming_variant_is_what_large_layers_run():
    """A layer large enough for the library to choose the streaming kernel by itself (six or more tile blocks per
    workgroup): equal to the direct kernel everywhere, and to the oracle on the first and the last image."""
    N, C, K, H, W = 6, 16, 32, 224, 224
    x, g = wl.make_custom(N, C, K, H, W, act="relu", wgt="gauss", seed=64)
    xd, gd = _x(x, wg.NHWC), _g(g, wg.NHWC)
    y = wg.winograd_conv2d_int8(xd, wg.winograd_filter_transform(gd, wg.NHWC, wg.LOSSLESS), wg.NHWC)
    assert torch.equal(y, wg.direct_conv2d_int8(xd, gd, wg.NHWC))
    for sl in (slice(0, 1), slice(N - 1, N)):
        assert np.array_equal(_y(y[sl], wg.NHWC), oracle.direct_conv2d(x[sl], g))
    ys = _y(wg.winograd_conv2d_int8(xd, wg.winograd_filter_transform(gd, wg.NHWC, wg.SCALED), wg.NHWC)[N - 1:], wg.NHWC)
    assert np.array_equal(ys, oracle.winograd_conv2d(x[N - 1:], g, oracle.SCALED)[0])


@pytest.mark.parametrize("path", PATHS, indirect=True)
def test_results_do_not_depend_on_workspace_contents_and_repeat_exactly(path):
    x, g = wl.make_custom(2, 24, 40, 14, 9, seed=40)
    packed = wg.winograd_filter_transform(_g(g, wg.NHWC), wg.NHWC, wg.LOSSLESS)
    xd = _x(x, wg.NHWC)
    ws = wg.make_workspace(2, 24, 14, 9, 40, wg.LOSSLESS)
    outs = []
    for fill in (0xA5, 0x00, 0xFF):
        ws.fill_(fill)
        outs.append(wg.winograd_conv2d_int8(xd, packed, wg.NHWC, workspace=ws).cpu().numpy())
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    assert np.array_equal(wl.from_nhwc(outs[0]), oracle.direct_conv2d(x, g))


@pytest.mark.parametrize("path", PATHS, indirect=True)
def test_output_canaries_survive_partial_tiles(path):
    """H, W not multiples of 4: stores are clipped to the image; guard elements around y stay intact."""
    x, g = wl.make_custom(1, 8, 6, 7, 5, seed=41)
    packed = wg.winograd_filter_transform(_g(g, wg.NCHW), wg.NCHW, wg.LOSSLESS)
    buf = torch.full((64 + 6 * 7 * 5 + 64,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    out = buf[64:64 + 6 * 7 * 5].view(1, 6, 7, 5)
    wg.winograd_conv2d_int8(_x(x, wg.NCHW), packed, wg.NCHW, out=out)
    assert np.array_equal(out.cpu().numpy(), oracle.direct_conv2d(x, g))
    assert (buf[:64] == 0x5A5A5A5A).all() and (buf[-64:] == 0x5A5A5A5A).all()


@pytest.mark.parametrize("path", PATHS, indirect=True)
def test_mismatched_blob_is_rejected_and_output_untouched(path):
    x, g = wl.make_custom(1, 8, 6, 8, 8, seed=42)
    packed = wg.winograd_filter_transform(_g(g, wg.NCHW), wg.NCHW, wg.LOSSLESS)
    wrong = wg.PackedFilter(packed.blob, packed.K, packed.C, wg.SCALED)
    with pytest.raises(wg.WinogradError):
        wrong.check()
    # the scaled-mode blob for this (K, C) is smaller, so the buffer is large enough to be read safely
    out = torch.full((1, 6, 8, 8), 77, dtype=torch.int32, device="cuda")
    wg.winograd_conv2d_int8(_x(x, wg.NCHW), wrong, wg.NCHW, out=out)
    assert (out == 77).all()
