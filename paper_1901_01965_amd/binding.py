"""Thin ctypes binding of libwinograd_mi355x.so: argument marshalling only.

Every step of the convolution runs in the library's HIP kernels.  PyTorch is
used for device memory (tensors' ``data_ptr()``) and for the current HIP
stream, nothing else.  There is no CPU or PyTorch fallback: if the shared
library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import torch

from .build import LIB_PATH

NCHW, NHWC = 0, 1
LOSSLESS, SCALED = 0, 1
MAX_CHANNELS = 896
_MODES = {"lossless": LOSSLESS, "scaled": SCALED, LOSSLESS: LOSSLESS, SCALED: SCALED}
_LAYOUTS = {"nchw": NCHW, "nhwc": NHWC, NCHW: NCHW, NHWC: NHWC}

_lib = None


class WinogradError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_string(status), status))


def load_library():
    """Load the in-tree HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "HIP library %s not found: run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(there is no fallback path)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    sigs = {
        "winograd_status_string": (ctypes.c_char_p, [i]),
        "winograd_num_activation_planes": (i, [i]),
        "winograd_num_filter_planes": (i, [i]),
        "winograd_debug_force_path": (i, [i]),
        "winograd_debug_stream_workgroups": (i, [i]),
        "winograd_debug_lossless_variant": (i, [i]),
        "winograd_debug_scaled_variant": (i, [i]),
        "winograd_debug_stream_variant": (i, [i]),
        "winograd_conv2d_path": (i, [i, i, i, i, i, i]),
        "winograd_debug_tile_decode": (i, [i, i, i, i, i, i, vp]),
        "winograd_packed_filter_bytes": (sz, [i, i, i]),
        "winograd_workspace_bytes": (sz, [i, i, i, i, i, i]),
        "winograd_filter_transform": (i, [vp, i, i, i, i, vp, sz, vp]),
        "winograd_packed_filter_check": (i, [vp, i, i, i, vp]),
        "winograd_conv2d_int8": (i, [vp, vp, vp, i, i, i, i, i, i, i, vp, sz, vp]),
        "winograd_conv2d_int8_requant": (i, [vp, vp, vp, i, i, i, i, i, i, i, i, i, i, vp]),
        "winograd_static_workspace_limit": (sz, []),
        "winograd_conv2d_int8_static_workspace": (i, [vp, vp, vp, i, i, i, i, i, i, i, vp]),
        "winograd_f2x2_packed_filter_bytes": (sz, [i, i, i]),
        "winograd_f2x2_filter_transform": (i, [vp, i, i, i, i, vp, sz, vp]),
        "winograd_f2x2_conv2d_int8": (i, [vp, vp, vp, i, i, i, i, i, i, i, vp]),
        "winograd_f2x2_debug_filter_operands": (i, [vp, i, i, i, vp, vp, vp]),
        "winograd_filter_transform_u8": (i, [vp, i, i, i, i, i, vp, sz, vp]),
        "winograd_conv2d_int8_act_scaled": (i, [vp, vp, vp, i, i, i, i, i, i, vp, vp]),
        "winograd_conv2d_u8": (i, [vp, i, vp, vp, i, i, i, i, i, i, i, vp]),
        "winograd_f2x2_filter_transform_u8": (i, [vp, i, i, i, i, i, vp, sz, vp]),
        "winograd_f2x2_conv2d_u8": (i, [vp, i, vp, vp, i, i, i, i, i, i, i, vp]),
        "winograd_f2x2_conv2d_int8_act_scaled": (i, [vp, vp, vp, i, i, i, i, i, i, vp, vp]),
        "winograd_f2x2_conv2d_int8_requant": (i, [vp, vp, vp, i, i, i, i, i, i, i, i, i, i, vp]),
        "winograd_conv2d_int8_enqueue_stage": (i, [vp, vp, vp, i, i, i, i, i, i, i, vp, sz, vp, i, i]),
        "direct_conv2d_int8": (i, [vp, vp, vp, i, i, i, i, i, i, vp]),
        "requant_relu_pool_int8": (i, [vp, vp, i, i, i, i, i, i, i, i, vp]),
        "winograd_debug_input_operands": (i, [vp, vp, i, i, i, i, i, i, vp, sz, vp]),
        "winograd_debug_filter_operands": (i, [vp, i, i, i, vp, vp, vp]),
        "winograd_debug_contraction": (i, [vp, vp, vp, i, i, i, i, i, i, i, vp, sz, vp]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


EXPORTED_SYMBOLS = (
    "winograd_status_string", "winograd_num_activation_planes", "winograd_num_filter_planes",
    "winograd_debug_force_path", "winograd_debug_stream_workgroups", "winograd_debug_lossless_variant", "winograd_debug_scaled_variant", "winograd_debug_stream_variant", "winograd_conv2d_path", "winograd_debug_tile_decode",
    "winograd_packed_filter_bytes", "winograd_workspace_bytes", "winograd_filter_transform",
    "winograd_packed_filter_check", "winograd_conv2d_int8", "winograd_conv2d_int8_requant",
    "winograd_static_workspace_limit", "winograd_conv2d_int8_static_workspace",
    "winograd_conv2d_int8_enqueue_stage",
    "direct_conv2d_int8", "requant_relu_pool_int8",
    "winograd_debug_input_operands", "winograd_debug_filter_operands", "winograd_debug_contraction",
    "winograd_f2x2_packed_filter_bytes", "winograd_f2x2_filter_transform", "winograd_f2x2_conv2d_int8",
    "winograd_f2x2_debug_filter_operands", "winograd_f2x2_filter_transform_u8", "winograd_f2x2_conv2d_u8",
    "winograd_f2x2_conv2d_int8_act_scaled", "winograd_f2x2_conv2d_int8_requant",
    "winograd_filter_transform_u8", "winograd_conv2d_u8", "winograd_conv2d_int8_act_scaled",
)


def status_string(status):
    return load_library().winograd_status_string(int(status)).decode()


def _check(status, where):
    if status != 0:
        raise WinogradError(status, where)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def _dims(x, layout):
    if layout == NCHW:
        N, C, H, W = x.shape
    else:
        N, H, W, C = x.shape
    return N, C, H, W


def _need(t, dtype, what):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of %s" % (what, dtype))


def _out(out, shape, dtype, device, what="out"):
    """A fresh output tensor, or the caller's after a check of its shape, type and contiguity: a kernel writes
    `shape` elements of `dtype` wherever the pointer leads."""
    if out is None:
        return torch.empty(shape, dtype=dtype, device=device)
    _need(out, dtype, what)
    if tuple(out.shape) != tuple(shape):
        raise ValueError("%s has shape %s, the call writes %s" % (what, tuple(out.shape), tuple(shape)))
    return out


def _match(packed, cls, C, what):
    """The blob must be of the right algorithm and made for the activation's channel count: the kernels only
    find a mismatch on the device, where all they can do is leave the output untouched."""
    if type(packed) is not cls:
        raise TypeError("%s needs a %s, got %s" % (what, cls.__name__, type(packed).__name__))
    if packed.C != C:
        raise ValueError("%s: the filters were packed for C = %d, the activations have C = %d" % (what, packed.C, C))


AUTO, STAGED, FUSED = 0, 1, 2


def force_path(path):
    """0: library's choice (the fused kernel), 1: staged three-kernel pipeline, 2: fused kernel."""
    _check(load_library().winograd_debug_force_path(int(path)), "winograd_debug_force_path")


def stream_workgroups(n):
    """Test hook: n > 0 = use the streaming variant of the single-kernel path with n workgroups per filter block."""
    _check(load_library().winograd_debug_stream_workgroups(int(n)), "winograd_debug_stream_workgroups")


def lossless_variant(v):
    """Test hook: 0 = library's choice of the lossless single-kernel form, 1 = limb-pair form wherever the layout
    allows, 2 = never the limb-pair form."""
    _check(load_library().winograd_debug_lossless_variant(int(v)), "winograd_debug_lossless_variant")


def stream_variant(v):
    """Test hook: 0 = library's choice of the streaming kernel's form, 1 = 64 filters per workgroup wherever a layer
    streams and the form applies (lossless mode, or one channel block), 2 = never."""
    _check(load_library().winograd_debug_stream_variant(int(v)), "winograd_debug_stream_variant")


def scaled_variant(v):
    """Test hook (both modes): 0 = library's choice, 1 = the role-specialised kernel with eight product waves (64 filters
    per workgroup) wherever the layout allows, 2 = never that form."""
    _check(load_library().winograd_debug_scaled_variant(int(v)), "winograd_debug_scaled_variant")


def conv2d_path(N, C, H, W, K, mode):
    """STAGED or FUSED: which implementation winograd_conv2d_int8 runs for this problem."""
    r = int(load_library().winograd_conv2d_path(N, C, H, W, K, _MODES[mode]))
    if r < 0:
        raise WinogradError(r, "winograd_conv2d_path")
    return r


def packed_filter_bytes(K, C, mode):
    return int(load_library().winograd_packed_filter_bytes(K, C, _MODES[mode]))


def workspace_bytes(N, C, H, W, K, mode):
    return int(load_library().winograd_workspace_bytes(N, C, H, W, K, _MODES[mode]))


class PackedFilter:
    """Device blob of Winograd-domain filters plus the (K, C, mode) it was made for."""

    def __init__(self, blob, K, C, mode):
        self.blob, self.K, self.C, self.mode = blob, K, C, mode

    def check(self):
        _check(load_library().winograd_packed_filter_check(_ptr(self.blob), self.K, self.C, self.mode, _stream()),
               "winograd_packed_filter_check")


def winograd_filter_transform(w, layout=NCHW, mode=LOSSLESS, blob=None):
    """w: int8 [K,C,3,3] (NCHW) or [K,3,3,C] (NHWC) on the GPU -> PackedFilter."""
    layout, mode = _LAYOUTS[layout], _MODES[mode]
    _need(w, torch.int8, "w")
    K = w.shape[0]
    C = w.shape[1] if layout == NCHW else w.shape[3]
    nbytes = packed_filter_bytes(K, C, mode)
    if nbytes == 0:
        _check(load_library().winograd_filter_transform(_ptr(w), K, C, layout, mode, None, 0, _stream()),
               "winograd_filter_transform")
    if blob is None:
        blob = torch.empty(nbytes, dtype=torch.uint8, device=w.device)
    _check(load_library().winograd_filter_transform(_ptr(w), K, C, layout, mode, _ptr(blob), blob.numel(), _stream()),
           "winograd_filter_transform")
    return PackedFilter(blob, K, C, mode)


class PackedFilterU8(PackedFilter):
    """Blob made from uint8 filters with a zero point (13-bit Winograd-domain values); goes with winograd_conv2d_u8."""


MAX_CHANNELS_U8 = 229


def winograd_filter_transform_u8(w, zero_point, layout=NCHW, mode=LOSSLESS):
    """w: uint8 [K,C,3,3] (NCHW) or [K,3,3,C] (NHWC) on the GPU, the filters being w - zero_point -> PackedFilterU8."""
    layout, mode = _LAYOUTS[layout], _MODES[mode]
    _need(w, torch.uint8, "w")
    K = w.shape[0]
    C = w.shape[1] if layout == NCHW else w.shape[3]
    nbytes = packed_filter_bytes(K, C, mode)
    blob = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=w.device)
    _check(load_library().winograd_filter_transform_u8(_ptr(w), int(zero_point), K, C, layout, mode, _ptr(blob), nbytes,
                                                       _stream()), "winograd_filter_transform_u8")
    return PackedFilterU8(blob, K, C, mode)


def winograd_conv2d_u8(x, zero_point, packed, layout=NCHW, out=None):
    """x: uint8 activations in `layout`, the values being x - zero_point; packed: PackedFilterU8.  int32 output."""
    layout = _LAYOUTS[layout]
    _need(x, torch.uint8, "x")
    N, C, H, W = _dims(x, layout)
    _match(packed, PackedFilterU8, C, "winograd_conv2d_u8")
    K = packed.K
    out = _out(out, (N, K, H, W) if layout == NCHW else (N, H, W, K), torch.int32, x.device)
    _check(load_library().winograd_conv2d_u8(_ptr(x), int(zero_point), _ptr(packed.blob), _ptr(out), N, C, H, W, K, layout,
                                             packed.mode, _stream()), "winograd_conv2d_u8")
    return out


def winograd_conv2d_int8_act_scaled(x, packed, layout=NCHW, out=None, want_table=False):
    """The complex F(4x4,3x3) path with the activations of every tile scaled into +-127 as well; packed: a SCALED
    blob of signed int8 filters.  want_table: also return the int32 [T, 26, 4] = (n, p, r, q) table the kernel
    derived per tile and free entry."""
    layout = _LAYOUTS[layout]
    _need(x, torch.int8, "x")
    N, C, H, W = _dims(x, layout)
    _match(packed, PackedFilter, C, "winograd_conv2d_int8_act_scaled")
    K = packed.K
    out = _out(out, (N, K, H, W) if layout == NCHW else (N, H, W, K), torch.int32, x.device)
    table = None
    if want_table:
        table = torch.empty((N * ((H + 3) // 4) * ((W + 3) // 4), 26, 4), dtype=torch.int32, device=x.device)
    _check(load_library().winograd_conv2d_int8_act_scaled(
        _ptr(x), _ptr(packed.blob), _ptr(out), N, C, H, W, K, layout,
        _ptr(table) if table is not None else ctypes.c_void_p(0), _stream()), "winograd_conv2d_int8_act_scaled")
    return (out, table) if want_table else out


def make_workspace(N, C, H, W, K, mode, device="cuda"):
    return torch.empty(workspace_bytes(N, C, H, W, K, mode), dtype=torch.uint8, device=device)


def winograd_conv2d_int8(x, packed, layout=NCHW, out=None, workspace=None):
    """x: int8 activations in `layout`; packed: PackedFilter.  Returns int32 output in `layout`."""
    layout = _LAYOUTS[layout]
    _need(x, torch.int8, "x")
    N, C, H, W = _dims(x, layout)
    _match(packed, PackedFilter, C, "winograd_conv2d_int8")
    K = packed.K
    if workspace is None:
        workspace = make_workspace(N, C, H, W, K, packed.mode, x.device)
    _need(workspace, torch.uint8, "workspace")
    out = _out(out, (N, K, H, W) if layout == NCHW else (N, H, W, K), torch.int32, x.device)
    _check(load_library().winograd_conv2d_int8(_ptr(x), _ptr(packed.blob), _ptr(out), N, C, H, W, K, layout,
                                               packed.mode, _ptr(workspace), workspace.numel(), _stream()),
           "winograd_conv2d_int8")
    return out


def static_workspace_limit():
    return int(load_library().winograd_static_workspace_limit())


def winograd_conv2d_int8_static_workspace(x, packed, layout=NCHW, out=None):
    """winograd_conv2d_int8's staged pipeline through the scratch buffer inside the library: the call itself
    allocates nothing (`out` given), and raises WG_ESMALLBUF beyond static_workspace_limit()."""
    layout = _LAYOUTS[layout]
    _need(x, torch.int8, "x")
    N, C, H, W = _dims(x, layout)
    _match(packed, PackedFilter, C, "winograd_conv2d_int8_static_workspace")
    K = packed.K
    out = _out(out, (N, K, H, W) if layout == NCHW else (N, H, W, K), torch.int32, x.device)
    _check(load_library().winograd_conv2d_int8_static_workspace(_ptr(x), _ptr(packed.blob), _ptr(out), N, C, H, W, K,
                                                                layout, packed.mode, _stream()),
           "winograd_conv2d_int8_static_workspace")
    return out


def winograd_conv2d_int8_requant(x, packed, shift, relu=True, pool=False, layout=NCHW, out=None):
    """Convolution with requantisation, ReLU and optional 2x2 max-pool applied before the store: int8 output in
    `layout` (H/2 x W/2 when pool), equal to winograd_conv2d_int8 followed by requant_relu_pool_int8."""
    layout = _LAYOUTS[layout]
    _need(x, torch.int8, "x")
    N, C, H, W = _dims(x, layout)
    _match(packed, PackedFilter, C, "winograd_conv2d_int8_requant")
    K = packed.K
    Ho, Wo = (H // 2, W // 2) if pool else (H, W)
    out = _out(out, (N, K, Ho, Wo) if layout == NCHW else (N, Ho, Wo, K), torch.int8, x.device)
    _check(load_library().winograd_conv2d_int8_requant(_ptr(x), _ptr(packed.blob), _ptr(out), N, C, H, W, K, layout,
                                                       packed.mode, int(shift), int(relu), int(pool), _stream()),
           "winograd_conv2d_int8_requant")
    return out


STAGE_NAMES = ("input_transform", "contraction", "output_transform", "fused_conv")


def enqueue_stage(x, packed, stage, iters, layout=NCHW, out=None, workspace=None):
    """Enqueues one kernel of winograd_conv2d_int8 (`stage`: an index into STAGE_NAMES) `iters` times on the current
    stream and returns at once; the caller times it with events on that stream."""
    layout = _LAYOUTS[layout]
    _need(x, torch.int8, "x")
    N, C, H, W = _dims(x, layout)
    _match(packed, PackedFilter, C, "enqueue_stage")
    K = packed.K
    if workspace is None:
        workspace = make_workspace(N, C, H, W, K, packed.mode, x.device)
    _need(workspace, torch.uint8, "workspace")
    out = _out(out, (N, K, H, W) if layout == NCHW else (N, H, W, K), torch.int32, x.device)
    _check(load_library().winograd_conv2d_int8_enqueue_stage(
        _ptr(x), _ptr(packed.blob), _ptr(out), N, C, H, W, K, layout, packed.mode, _ptr(workspace),
        workspace.numel(), _stream(), int(stage), int(iters)), "winograd_conv2d_int8_enqueue_stage")
    return out


def direct_conv2d_int8(x, w, layout=NCHW, out=None):
    layout = _LAYOUTS[layout]
    _need(x, torch.int8, "x")
    _need(w, torch.int8, "w")
    N, C, H, W = _dims(x, layout)
    K = w.shape[0]
    if tuple(w.shape) != ((K, C, 3, 3) if layout == NCHW else (K, 3, 3, C)):
        raise ValueError("w has shape %s, which does not fit activations with C = %d" % (tuple(w.shape), C))
    out = _out(out, (N, K, H, W) if layout == NCHW else (N, H, W, K), torch.int32, x.device)
    _check(load_library().direct_conv2d_int8(_ptr(x), _ptr(w), _ptr(out), N, C, H, W, K, layout, _stream()),
           "direct_conv2d_int8")
    return out


def requant_relu_pool_int8(y, shift, relu=True, pool=False, layout=NCHW, out=None):
    layout = _LAYOUTS[layout]
    _need(y, torch.int32, "y")
    N, K, H, W = _dims(y, layout)
    Ho, Wo = (H // 2, W // 2) if pool else (H, W)
    out = _out(out, (N, K, Ho, Wo) if layout == NCHW else (N, Ho, Wo, K), torch.int8, y.device)
    _check(load_library().requant_relu_pool_int8(_ptr(y), _ptr(out), N, K, H, W, layout, int(shift), int(relu),
                                                 int(pool), _stream()), "requant_relu_pool_int8")
    return out


def debug_input_operands(x, layout=NCHW, mode=LOSSLESS):
    """int8 [planes, T, C]: the operand planes the input transform hands to the contraction."""
    layout, mode = _LAYOUTS[layout], _MODES[mode]
    _need(x, torch.int8, "x")
    N, C, H, W = _dims(x, layout)
    lib = load_library()
    T = N * ((H + 3) // 4) * ((W + 3) // 4)
    out = torch.empty((lib.winograd_num_activation_planes(mode), T, C), dtype=torch.int8, device=x.device)
    ws = make_workspace(N, C, H, W, 1, mode, x.device)
    _check(lib.winograd_debug_input_operands(_ptr(x), _ptr(out), N, C, H, W, layout, mode, _ptr(ws), ws.numel(),
                                             _stream()), "winograd_debug_input_operands")
    return out


def debug_filter_operands(packed):
    """(int8 [planes, K, C], int32 [K, 26, 4]) unpacked from a PackedFilter."""
    lib = load_library()
    planes = torch.empty((lib.winograd_num_filter_planes(packed.mode), packed.K, packed.C), dtype=torch.int8,
                         device=packed.blob.device)
    table = torch.empty((packed.K, 26, 4), dtype=torch.int32, device=packed.blob.device)
    _check(lib.winograd_debug_filter_operands(_ptr(packed.blob), packed.K, packed.C, packed.mode, _ptr(planes),
                                              _ptr(table), _stream()), "winograd_debug_filter_operands")
    return planes, table


def debug_contraction(x, packed, layout=NCHW):
    """int32 [36, T, K]: the Winograd-domain accumulators after contraction (and inverse scaling)."""
    layout = _LAYOUTS[layout]
    _need(x, torch.int8, "x")
    N, C, H, W = _dims(x, layout)
    _match(packed, PackedFilter, C, "debug_contraction")
    T = N * ((H + 3) // 4) * ((W + 3) // 4)
    out = torch.empty((36, T, packed.K), dtype=torch.int32, device=x.device)
    ws = make_workspace(N, C, H, W, packed.K, packed.mode, x.device)
    _check(load_library().winograd_debug_contraction(_ptr(x), _ptr(packed.blob), _ptr(out), N, C, H, W, packed.K,
                                                     layout, packed.mode, _ptr(ws), ws.numel(), _stream()),
           "winograd_debug_contraction")
    return out


# ---- rational F(2x2,3x3) --------------------------------------------------------------------------------------

class F2x2PackedFilter:
    """Winograd-domain filters of the F(2x2,3x3) path: device blob plus the (K, C, mode) it was made for."""

    def __init__(self, blob, K, C, mode):
        self.blob, self.K, self.C, self.mode = blob, K, C, mode


def f2x2_filter_transform(w, layout=NCHW, mode=LOSSLESS, zero_point=None):
    """w: int8 filters, or uint8 filters with their zero point (values w - zero_point)."""
    layout = _LAYOUTS[layout]
    _need(w, torch.int8 if zero_point is None else torch.uint8, "w")
    K = w.shape[0]
    C = w.shape[1] if layout == NCHW else w.shape[3]
    nbytes = load_library().winograd_f2x2_packed_filter_bytes(K, C, mode)
    if nbytes == 0:
        raise WinogradError(-1, "winograd_f2x2_packed_filter_bytes")
    blob = torch.empty(nbytes, dtype=torch.uint8, device=w.device)
    if zero_point is None:
        _check(load_library().winograd_f2x2_filter_transform(_ptr(w), K, C, layout, mode, _ptr(blob), nbytes, _stream()),
               "winograd_f2x2_filter_transform")
    else:
        _check(load_library().winograd_f2x2_filter_transform_u8(_ptr(w), int(zero_point), K, C, layout, mode, _ptr(blob),
                                                                nbytes, _stream()), "winograd_f2x2_filter_transform_u8")
    return F2x2PackedFilter(blob, K, C, mode)


def f2x2_conv2d_int8(x, packed, layout=NCHW, out=None, zero_point=None):
    """x: int8 activations, or uint8 activations with their zero point (values x - zero_point)."""
    layout = _LAYOUTS[layout]
    _need(x, torch.int8 if zero_point is None else torch.uint8, "x")
    N, C, H, W = _dims(x, layout)
    _match(packed, F2x2PackedFilter, C, "f2x2_conv2d_int8")
    K = packed.K
    out = _out(out, (N, K, H, W) if layout == NCHW else (N, H, W, K), torch.int32, x.device)
    if zero_point is None:
        _check(load_library().winograd_f2x2_conv2d_int8(_ptr(x), _ptr(packed.blob), _ptr(out), N, C, H, W, K, layout,
                                                        packed.mode, _stream()), "winograd_f2x2_conv2d_int8")
    else:
        _check(load_library().winograd_f2x2_conv2d_u8(_ptr(x), int(zero_point), _ptr(packed.blob), _ptr(out), N, C, H, W, K,
                                                      layout, packed.mode, _stream()), "winograd_f2x2_conv2d_u8")
    return out


def f2x2_conv2d_int8_requant(x, packed, shift, relu=True, pool=False, layout=NCHW, out=None):
    """F(2x2,3x3) convolution with requantisation, ReLU and optional 2x2 max-pool before the store: int8 output."""
    layout = _LAYOUTS[layout]
    _need(x, torch.int8, "x")
    N, C, H, W = _dims(x, layout)
    _match(packed, F2x2PackedFilter, C, "f2x2_conv2d_int8_requant")
    K = packed.K
    Ho, Wo = (H // 2, W // 2) if pool else (H, W)
    out = _out(out, (N, K, Ho, Wo) if layout == NCHW else (N, Ho, Wo, K), torch.int8, x.device)
    _check(load_library().winograd_f2x2_conv2d_int8_requant(_ptr(x), _ptr(packed.blob), _ptr(out), N, C, H, W, K, layout,
                                                            packed.mode, int(shift), int(bool(relu)), int(bool(pool)),
                                                            _stream()), "winograd_f2x2_conv2d_int8_requant")
    return out


def f2x2_conv2d_int8_act_scaled(x, packed, layout=NCHW, out=None, want_table=False):
    """F(2x2,3x3) with the activations of every tile scaled into +-127 as well; packed: a SCALED blob of signed int8
    filters.  want_table: also return the int32 [T, 16, 4] = (n, p, r, q) table the kernel derived per tile."""
    layout = _LAYOUTS[layout]
    _need(x, torch.int8, "x")
    N, C, H, W = _dims(x, layout)
    _match(packed, F2x2PackedFilter, C, "f2x2_conv2d_int8_act_scaled")
    K = packed.K
    out = _out(out, (N, K, H, W) if layout == NCHW else (N, H, W, K), torch.int32, x.device)
    table = None
    if want_table:
        table = torch.empty((N * ((H + 1) // 2) * ((W + 1) // 2), 16, 4), dtype=torch.int32, device=x.device)
    _check(load_library().winograd_f2x2_conv2d_int8_act_scaled(
        _ptr(x), _ptr(packed.blob), _ptr(out), N, C, H, W, K, layout,
        _ptr(table) if table is not None else ctypes.c_void_p(0), _stream()), "winograd_f2x2_conv2d_int8_act_scaled")
    return (out, table) if want_table else out


def f2x2_debug_filter_operands(packed):
    """(planes int8 [planes, K, C], table int32 [K, 16, 4] = (n, p, r, q)) as the blob holds them."""
    planes = 32 if packed.mode == LOSSLESS else 16
    dense = torch.empty((planes, packed.K, packed.C), dtype=torch.int8, device=packed.blob.device)
    table = torch.empty((packed.K, 16, 4), dtype=torch.int32, device=packed.blob.device)
    _check(load_library().winograd_f2x2_debug_filter_operands(_ptr(packed.blob), packed.K, packed.C, packed.mode,
                                                              _ptr(dense), _ptr(table), _stream()),
           "winograd_f2x2_debug_filter_operands")
    return dense, table
