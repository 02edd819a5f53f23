"""Integer complex-Winograd F(4x4,3x3) convolution for MI355X (gfx950).

The product is the HIP library under ``csrc/`` behind the C ABI declared in
``include/winograd_c.h``; ``binding`` marshals PyTorch device tensors into it and
``workloads`` makes the seeded synthetic inputs.  Importing the package does
not load the library; the first call does, and fails loudly if it is absent.
"""
from . import workloads  # noqa: F401
from .binding import (  # noqa: F401
    LOSSLESS, SCALED, NCHW, NHWC, MAX_CHANNELS, PackedFilter, WinogradError,
    winograd_filter_transform, winograd_conv2d_int8, winograd_conv2d_int8_requant, direct_conv2d_int8,
    winograd_conv2d_int8_static_workspace, static_workspace_limit,
    winograd_filter_transform_u8, winograd_conv2d_u8, winograd_conv2d_int8_act_scaled, PackedFilterU8, MAX_CHANNELS_U8,
    requant_relu_pool_int8,
    packed_filter_bytes, workspace_bytes, make_workspace, load_library,
    f2x2_filter_transform, f2x2_conv2d_int8, f2x2_debug_filter_operands, F2x2PackedFilter, f2x2_conv2d_int8_act_scaled, f2x2_conv2d_int8_requant,
    debug_input_operands, debug_filter_operands, debug_contraction, enqueue_stage, STAGE_NAMES, force_path, stream_workgroups, lossless_variant, scaled_variant, stream_variant, conv2d_path, AUTO, STAGED, FUSED,
)
