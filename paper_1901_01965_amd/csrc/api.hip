// The C ABI: argument validation on the host, then the stage launchers.
// Nothing here allocates, and nothing synchronises except winograd_packed_filter_check.
#include <atomic>

#include "api_checks.h"

using namespace wg;

namespace {

// 0: the library's choice (the fused kernel: on every measured shape it is at least as fast as
// the staged pipeline, which moves the transformed activations and the accumulator planes
// through memory); 1: always the staged three-kernel pipeline; 2: always the fused kernel.
std::atomic<int> g_forced_path{0};

bool use_fused() { return g_forced_path.load(std::memory_order_relaxed) != 1; }

}  // namespace

extern "C" {

const char* winograd_status_string(int status) {
    switch (status) {
        case WG_OK: return "ok";
        case WG_EINVAL: return "invalid argument (null or misaligned pointer, non-positive size, unknown enum)";
        case WG_EUNSUPPORTED: return "unsupported problem (too many input channels or tensor too large)";
        case WG_ESMALLBUF: return "buffer smaller than the size query reports";
        case WG_EBLOB: return "packed filter blob does not match (K, C, mode)";
        case WG_ERUNTIME: return "HIP runtime error";
        default: return "unknown status";
    }
}

int winograd_num_activation_planes(int mode) { return valid_mode(mode) ? num_activation_planes(mode) : 0; }
int winograd_num_filter_planes(int mode) { return valid_mode(mode) ? num_filter_planes(mode) : 0; }

size_t winograd_packed_filter_bytes(int K, int C, int mode) {
    if (check_filter_shape(K, C) != WG_OK || !valid_mode(mode)) return 0;
    return blob_layout(ceil_div(K, kFilterPad) * kFilterPad, C, mode).total;
}

size_t winograd_workspace_bytes(int N, int C, int H, int W, int K, int mode) {
    if (check_shape(N, C, H, W, K) != WG_OK || !valid_mode(mode)) return 0;
    return workspace_layout(make_problem(N, C, H, W, K), mode).total;
}

int winograd_filter_transform(const int8_t* w_dev, int K, int C, int layout, int mode, void* packed_dev,
                              size_t packed_bytes, void* hip_stream) {
    if (!w_dev || !packed_dev || !valid_layout(layout) || !valid_mode(mode)) return WG_EINVAL;
    if (int st = check_filter_shape(K, C)) return st;
    if (!aligned(w_dev, 4) || !aligned(packed_dev, 256)) return WG_EINVAL;
    if (packed_bytes < winograd_packed_filter_bytes(K, C, mode)) return WG_ESMALLBUF;
    return status_of(launch_filter_transform(w_dev, 0, 0, K, C, layout, mode, packed_dev,
                                             static_cast<hipStream_t>(hip_stream)));
}

int winograd_filter_transform_u8(const uint8_t* w_dev, int zero_point, int K, int C, int layout, int mode, void* packed_dev,
                                 size_t packed_bytes, void* hip_stream) {
    if (!w_dev || !packed_dev || !valid_layout(layout) || !valid_mode(mode)) return WG_EINVAL;
    if (zero_point < 0 || zero_point > 255) return WG_EINVAL;
    if (int st = check_filter_shape(K, C)) return st;
    if (C > kMaxChannelsInt9) return WG_EUNSUPPORTED;
    if (!aligned(w_dev, 4) || !aligned(packed_dev, 256)) return WG_EINVAL;
    if (packed_bytes < winograd_packed_filter_bytes(K, C, mode)) return WG_ESMALLBUF;
    return status_of(launch_filter_transform(reinterpret_cast<const int8_t*>(w_dev), 1, zero_point, K, C, layout, mode,
                                             packed_dev, static_cast<hipStream_t>(hip_stream)));
}

int winograd_conv2d_u8(const uint8_t* x_dev, int zero_point, const void* packed_dev, int32_t* y_dev, int N, int C, int H,
                       int W, int K, int layout, int mode, void* hip_stream) {
    if (!x_dev || !packed_dev || !y_dev || !valid_layout(layout) || !valid_mode(mode)) return WG_EINVAL;
    if (zero_point < 0 || zero_point > 255) return WG_EINVAL;
    if (int st = check_shape(N, C, H, W, K)) return st;
    if (C > kMaxChannelsInt9) return WG_EUNSUPPORTED;
    if (!aligned(x_dev, 4) || !aligned(y_dev, 4) || !aligned(packed_dev, 256)) return WG_EINVAL;
    return status_of(launch_fused_conv_u8(x_dev, zero_point, packed_dev, y_dev, make_problem(N, C, H, W, K), layout, mode,
                                          static_cast<hipStream_t>(hip_stream)));
}

int winograd_conv2d_int8_act_scaled(const int8_t* x_dev, const void* packed_dev, int32_t* y_dev, int N, int C, int H, int W,
                                    int K, int layout, int32_t* act_table_dev, void* hip_stream) {
    if (!x_dev || !packed_dev || !y_dev || !valid_layout(layout)) return WG_EINVAL;
    if (int st = check_shape(N, C, H, W, K)) return st;
    if (!aligned(x_dev, 4) || !aligned(y_dev, 4) || !aligned(packed_dev, 256)) return WG_EINVAL;
    if (act_table_dev && !aligned(act_table_dev, 16)) return WG_EINVAL;
    return status_of(launch_fused_conv_act_scaled(x_dev, packed_dev, y_dev, act_table_dev, make_problem(N, C, H, W, K), layout,
                                                  static_cast<hipStream_t>(hip_stream)));
}

int winograd_packed_filter_check(const void* packed_dev, int K, int C, int mode, void* hip_stream) {
    if (!packed_dev || !valid_mode(mode)) return WG_EINVAL;
    if (int st = check_filter_shape(K, C)) return st;
    BlobHeader h;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (hipMemcpyAsync(&h, packed_dev, sizeof h, hipMemcpyDeviceToHost, s) != hipSuccess) return WG_ERUNTIME;
    if (hipStreamSynchronize(s) != hipSuccess) return WG_ERUNTIME;
    const bool ok = (h.magic == kBlobMagic || h.magic == kBlobMagicInt9) && h.version == kBlobVersion && h.K == K && h.C == C && h.mode == mode;
    return ok ? WG_OK : WG_EBLOB;
}

static int check_conv_args(const void* x, const void* packed, const void* y, int N, int C, int H, int W, int K,
                           int layout, int mode, const void* ws, size_t ws_bytes) {
    if (!x || !packed || !y || !ws || !valid_layout(layout) || !valid_mode(mode)) return WG_EINVAL;
    if (int st = check_shape(N, C, H, W, K)) return st;
    if (!aligned(x, 4) || !aligned(y, 4) || !aligned(packed, 256) || !aligned(ws, 256)) return WG_EINVAL;
    if (ws_bytes < winograd_workspace_bytes(N, C, H, W, K, mode)) return WG_ESMALLBUF;
    return WG_OK;
}

int winograd_conv2d_int8(const int8_t* x_dev, const void* packed_dev, int32_t* y_dev, int N, int C, int H,
                         int W, int K, int layout, int mode, void* workspace_dev, size_t workspace_bytes,
                         void* hip_stream) {
    if (int st = check_conv_args(x_dev, packed_dev, y_dev, N, C, H, W, K, layout, mode, workspace_dev,
                                 workspace_bytes))
        return st;
    const Problem p = make_problem(N, C, H, W, K);
    const WorkspaceLayout wl = workspace_layout(p, mode);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (use_fused()) return status_of(launch_fused_conv(x_dev, packed_dev, y_dev, p, layout, mode, no_int8_epilogue(), s));
    int8_t* V = static_cast<int8_t*>(workspace_dev) + wl.v_off;
    int32_t* M = reinterpret_cast<int32_t*>(static_cast<uint8_t*>(workspace_dev) + wl.m_off);
    if (int st = status_of(launch_input_transform(x_dev, p, layout, mode, V, s))) return st;
    if (int st = status_of(launch_contraction(V, packed_dev, M, p, mode, s))) return st;
    return status_of(launch_output_transform(M, packed_dev, y_dev, p, layout, mode, s));
}

int winograd_conv2d_int8_requant(const int8_t* x_dev, const void* packed_dev, int8_t* out_dev, int N, int C, int H,
                                 int W, int K, int layout, int mode, int shift, int relu, int pool,
                                 void* hip_stream) {
    if (!x_dev || !packed_dev || !out_dev || !valid_layout(layout) || !valid_mode(mode)) return WG_EINVAL;
    if (shift < 0 || shift > 31) return WG_EINVAL;
    if (int st = check_shape(N, C, H, W, K)) return st;
    if (!aligned(x_dev, 4) || !aligned(out_dev, 4) || !aligned(packed_dev, 256)) return WG_EINVAL;
    if (pool && ((H | W) & 1)) return WG_EUNSUPPORTED;
    const Problem p = make_problem(N, C, H, W, K);
    return status_of(launch_fused_conv(x_dev, packed_dev, nullptr, p, layout, mode,
                                       make_int8_epilogue(out_dev, shift, relu != 0, pool != 0),
                                       static_cast<hipStream_t>(hip_stream)));
}

size_t winograd_f2x2_packed_filter_bytes(int K, int C, int mode) {
    if (check_filter_shape(K, C) != WG_OK || !valid_mode(mode)) return 0;
    return f2_blob_layout(ceil_div(K, kFilterPad) * kFilterPad, C, mode).total;
}

static int f2_filter_transform(const void* w_dev, int is_unsigned, int zero_point, int K, int C, int layout, int mode,
                               void* packed_dev, size_t packed_bytes, void* hip_stream) {
    if (!w_dev || !packed_dev || !valid_layout(layout) || !valid_mode(mode)) return WG_EINVAL;
    if (is_unsigned && (zero_point < 0 || zero_point > 255)) return WG_EINVAL;
    if (int st = check_filter_shape(K, C)) return st;
    if (!aligned(w_dev, 4) || !aligned(packed_dev, 256)) return WG_EINVAL;
    if (packed_bytes < winograd_f2x2_packed_filter_bytes(K, C, mode)) return WG_ESMALLBUF;
    return status_of(launch_f2_filter_transform(static_cast<const int8_t*>(w_dev), is_unsigned, zero_point, K, C, layout,
                                                mode, packed_dev, static_cast<hipStream_t>(hip_stream)));
}

static int f2_conv2d(const void* x_dev, int is_unsigned, int zero_point, const void* packed_dev, int32_t* y_dev, int N,
                     int C, int H, int W, int K, int layout, int mode, void* hip_stream) {
    if (!x_dev || !packed_dev || !y_dev || !valid_layout(layout) || !valid_mode(mode)) return WG_EINVAL;
    if (is_unsigned && (zero_point < 0 || zero_point > 255)) return WG_EINVAL;
    if (int st = check_shape(N, C, H, W, K)) return st;
    const long long tiles = (long long)N * ((H + 1) / 2) * ((W + 1) / 2);   // 2x2 tiles: four times as many
    if (tiles + kTilePad > kIndexLimit / 64) return WG_EUNSUPPORTED;
    if (!aligned(x_dev, 4) || !aligned(y_dev, 4) || !aligned(packed_dev, 256)) return WG_EINVAL;
    return status_of(launch_f2_conv(static_cast<const int8_t*>(x_dev), is_unsigned, zero_point, packed_dev, y_dev,
                                    make_problem_f2(N, C, H, W, K), layout, mode, no_int8_epilogue(),
                                    static_cast<hipStream_t>(hip_stream)));
}

int winograd_f2x2_conv2d_int8_requant(const int8_t* x_dev, const void* packed_dev, int8_t* out_dev, int N, int C, int H,
                                      int W, int K, int layout, int mode, int shift, int relu, int pool,
                                      void* hip_stream) {
    if (!x_dev || !packed_dev || !out_dev || !valid_layout(layout) || !valid_mode(mode)) return WG_EINVAL;
    if (shift < 0 || shift > 31) return WG_EINVAL;
    if (int st = check_shape(N, C, H, W, K)) return st;
    const long long tiles = (long long)N * ((H + 1) / 2) * ((W + 1) / 2);
    if (tiles + kTilePad > kIndexLimit / 64) return WG_EUNSUPPORTED;
    if (!aligned(x_dev, 4) || !aligned(out_dev, 4) || !aligned(packed_dev, 256)) return WG_EINVAL;
    if (pool && ((H | W) & 1)) return WG_EUNSUPPORTED;
    return status_of(launch_f2_conv(x_dev, 0, 0, packed_dev, nullptr, make_problem_f2(N, C, H, W, K), layout, mode,
                                    make_int8_epilogue(out_dev, shift, relu != 0, pool != 0),
                                    static_cast<hipStream_t>(hip_stream)));
}

int winograd_f2x2_filter_transform(const int8_t* w_dev, int K, int C, int layout, int mode, void* packed_dev,
                                   size_t packed_bytes, void* hip_stream) {
    return f2_filter_transform(w_dev, 0, 0, K, C, layout, mode, packed_dev, packed_bytes, hip_stream);
}

int winograd_f2x2_filter_transform_u8(const uint8_t* w_dev, int zero_point, int K, int C, int layout, int mode,
                                      void* packed_dev, size_t packed_bytes, void* hip_stream) {
    return f2_filter_transform(w_dev, 1, zero_point, K, C, layout, mode, packed_dev, packed_bytes, hip_stream);
}

int winograd_f2x2_conv2d_int8(const int8_t* x_dev, const void* packed_dev, int32_t* y_dev, int N, int C, int H,
                              int W, int K, int layout, int mode, void* hip_stream) {
    return f2_conv2d(x_dev, 0, 0, packed_dev, y_dev, N, C, H, W, K, layout, mode, hip_stream);
}

int winograd_f2x2_conv2d_u8(const uint8_t* x_dev, int zero_point, const void* packed_dev, int32_t* y_dev, int N, int C,
                            int H, int W, int K, int layout, int mode, void* hip_stream) {
    return f2_conv2d(x_dev, 1, zero_point, packed_dev, y_dev, N, C, H, W, K, layout, mode, hip_stream);
}

int winograd_f2x2_conv2d_int8_act_scaled(const int8_t* x_dev, const void* packed_dev, int32_t* y_dev, int N, int C,
                                         int H, int W, int K, int layout, int32_t* act_table_dev, void* hip_stream) {
    if (!x_dev || !packed_dev || !y_dev || !valid_layout(layout)) return WG_EINVAL;
    if (int st = check_shape(N, C, H, W, K)) return st;
    const long long tiles = (long long)N * ((H + 1) / 2) * ((W + 1) / 2);
    if (tiles + kTilePad > kIndexLimit / 64) return WG_EUNSUPPORTED;
    if (!aligned(x_dev, 4) || !aligned(y_dev, 4) || !aligned(packed_dev, 256)) return WG_EINVAL;
    if (act_table_dev && !aligned(act_table_dev, 16)) return WG_EINVAL;
    return status_of(launch_f2_conv_act_scaled(x_dev, packed_dev, y_dev, act_table_dev, make_problem_f2(N, C, H, W, K),
                                               layout, static_cast<hipStream_t>(hip_stream)));
}

int winograd_f2x2_debug_filter_operands(const void* packed_dev, int K, int C, int mode, int8_t* planes_dev,
                                        int32_t* table_dev, void* hip_stream) {
    if (!packed_dev || !planes_dev || !table_dev || !valid_mode(mode)) return WG_EINVAL;
    if (int st = check_filter_shape(K, C)) return st;
    return status_of(launch_f2_unpack_filter_planes(packed_dev, planes_dev, table_dev, K, C, mode,
                                                    static_cast<hipStream_t>(hip_stream)));
}

int winograd_conv2d_path(int N, int C, int H, int W, int K, int mode) {
    if (!valid_mode(mode)) return WG_EINVAL;
    if (int st = check_shape(N, C, H, W, K)) return st;
    return use_fused() ? 2 : 1;
}

int winograd_debug_tile_decode(int N, int C, int H, int W, int K, int t, int* out3_host) {
    if (!out3_host || t < 0) return WG_EINVAL;
    if (int st = check_shape(N, C, H, W, K)) return st;
    const Problem p = make_problem(N, C, H, W, K);
    if (t >= p.T) return WG_EINVAL;
    decode_tile(p, t, out3_host[0], out3_host[1], out3_host[2]);
    return WG_OK;
}

int winograd_debug_stream_workgroups(int n) {
    if (n < 0) return WG_EINVAL;
    set_stream_workgroups(n);
    return WG_OK;
}

int winograd_debug_lossless_variant(int variant) {
    if (variant < 0 || variant > 2) return WG_EINVAL;
    set_lossless_variant(variant);
    return WG_OK;
}

int winograd_debug_scaled_variant(int variant) {
    if (variant < 0 || variant > 2) return WG_EINVAL;
    set_scaled_variant(variant);
    return WG_OK;
}

int winograd_debug_stream_variant(int variant) {
    if (variant < 0 || variant > 2) return WG_EINVAL;
    set_stream_variant(variant);
    return WG_OK;
}

int winograd_debug_force_path(int path) {
    if (path < 0 || path > 2) return WG_EINVAL;
    g_forced_path.store(path, std::memory_order_relaxed);
    return WG_OK;
}

int winograd_conv2d_int8_enqueue_stage(const int8_t* x_dev, const void* packed_dev, int32_t* y_dev, int N, int C,
                                       int H, int W, int K, int layout, int mode, void* workspace_dev,
                                       size_t workspace_bytes, void* hip_stream, int stage, int iters) {
    if (stage < 0 || stage > 3 || iters < 1) return WG_EINVAL;
    if (int st = check_conv_args(x_dev, packed_dev, y_dev, N, C, H, W, K, layout, mode, workspace_dev,
                                 workspace_bytes))
        return st;
    const Problem p = make_problem(N, C, H, W, K);
    const WorkspaceLayout wl = workspace_layout(p, mode);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int8_t* V = static_cast<int8_t*>(workspace_dev) + wl.v_off;
    int32_t* M = reinterpret_cast<int32_t*>(static_cast<uint8_t*>(workspace_dev) + wl.m_off);
    hipError_t e = hipSuccess;
    for (int i = 0; i < iters && e == hipSuccess; ++i) {
        if (stage == 0)      e = launch_input_transform(x_dev, p, layout, mode, V, s);
        else if (stage == 1) e = launch_contraction(V, packed_dev, M, p, mode, s);
        else if (stage == 2) e = launch_output_transform(M, packed_dev, y_dev, p, layout, mode, s);
        else                 e = launch_fused_conv(x_dev, packed_dev, y_dev, p, layout, mode, no_int8_epilogue(), s);
    }
    return status_of(e);
}

int direct_conv2d_int8(const int8_t* x_dev, const int8_t* w_dev, int32_t* y_dev, int N, int C, int H, int W,
                       int K, int layout, void* hip_stream) {
    if (!x_dev || !w_dev || !y_dev || !valid_layout(layout)) return WG_EINVAL;
    if (int st = check_shape(N, C, H, W, K)) return st;
    if (!aligned(x_dev, 4) || !aligned(w_dev, 4) || !aligned(y_dev, 4)) return WG_EINVAL;
    return status_of(launch_direct_conv(x_dev, w_dev, y_dev, make_problem(N, C, H, W, K), layout,
                                        static_cast<hipStream_t>(hip_stream)));
}

int requant_relu_pool_int8(const int32_t* y_dev, int8_t* out_dev, int N, int K, int H, int W, int layout,
                           int shift, int relu, int pool, void* hip_stream) {
    if (!y_dev || !out_dev || !valid_layout(layout)) return WG_EINVAL;
    if (N <= 0 || K <= 0 || H <= 0 || W <= 0 || shift < 0 || shift > 31) return WG_EINVAL;
    if (!aligned(y_dev, 4)) return WG_EINVAL;
    if (pool && ((H | W) & 1)) return WG_EUNSUPPORTED;
    if ((long long)N * K > kIndexLimit / ((long long)H * W)) return WG_EUNSUPPORTED;
    return status_of(launch_requant_relu_pool(y_dev, out_dev, N, K, H, W, layout, shift, relu != 0, pool != 0,
                                              static_cast<hipStream_t>(hip_stream)));
}

int winograd_debug_input_operands(const int8_t* x_dev, int8_t* planes_dev, int N, int C, int H, int W,
                                  int layout, int mode, void* workspace_dev, size_t workspace_bytes,
                                  void* hip_stream) {
    if (!x_dev || !planes_dev || !workspace_dev || !valid_layout(layout) || !valid_mode(mode)) return WG_EINVAL;
    if (int st = check_shape(N, C, H, W, 1)) return st;
    if (!aligned(x_dev, 4) || !aligned(workspace_dev, 256)) return WG_EINVAL;
    if (workspace_bytes < winograd_workspace_bytes(N, C, H, W, 1, mode)) return WG_ESMALLBUF;
    const Problem p = make_problem(N, C, H, W, 1);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int8_t* V = static_cast<int8_t*>(workspace_dev);
    if (int st = status_of(launch_input_transform(x_dev, p, layout, mode, V, s))) return st;
    return status_of(launch_unpack_activation_planes(V, planes_dev, p, mode, s));
}

int winograd_debug_filter_operands(const void* packed_dev, int K, int C, int mode, int8_t* planes_dev,
                                   int32_t* table_dev, void* hip_stream) {
    if (!packed_dev || !planes_dev || !table_dev || !valid_mode(mode)) return WG_EINVAL;
    if (int st = check_filter_shape(K, C)) return st;
    if (!aligned(packed_dev, 256) || !aligned(table_dev, 4)) return WG_EINVAL;
    return status_of(launch_unpack_filter_planes(packed_dev, planes_dev, table_dev, K, C, mode,
                                                 static_cast<hipStream_t>(hip_stream)));
}

int winograd_debug_contraction(const int8_t* x_dev, const void* packed_dev, int32_t* m_dev, int N, int C,
                               int H, int W, int K, int layout, int mode, void* workspace_dev,
                               size_t workspace_bytes, void* hip_stream) {
    if (int st = check_conv_args(x_dev, packed_dev, m_dev, N, C, H, W, K, layout, mode, workspace_dev,
                                 workspace_bytes))
        return st;
    const Problem p = make_problem(N, C, H, W, K);
    const WorkspaceLayout wl = workspace_layout(p, mode);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int8_t* V = static_cast<int8_t*>(workspace_dev) + wl.v_off;
    int32_t* M = reinterpret_cast<int32_t*>(static_cast<uint8_t*>(workspace_dev) + wl.m_off);
    if (int st = status_of(launch_input_transform(x_dev, p, layout, mode, V, s))) return st;
    if (int st = status_of(launch_contraction(V, packed_dev, M, p, mode, s))) return st;
    return status_of(launch_unpack_accumulators(M, m_dev, p, mode, s));
}

}  // extern "C"
