// Internal declarations shared by the HIP translation units of the library:
// problem geometry, HBM layouts of the packed filter blob and the workspace,
// the numbering of the free Winograd-domain entries, and the stage launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

#include "winograd_c.h"

namespace wg {

// ---- geometry ---------------------------------------------------------------
constexpr int kCBlock = 64;      // input channels per operand row (bytes per row)
constexpr int kTilePad = 64;     // tile count is padded to a multiple of this
constexpr int kFilterPad = 64;   // filter count is padded to a multiple of this
constexpr int kEntries = 26;     // free entries of a transformed 6x6 tile (Section 3.4)
constexpr int kRealEntries = 16;
constexpr int kAccPlanes = 36;   // 16 real + 10 * (Re, Im): the planes the output transform consumes
constexpr int kMaxWorkspacePlanes = 46;   // lossless keeps the three products of a complex entry apart
constexpr int kWeightRange = 127;  // spatial range of signed int8 filters, the target of the scaling

// Division of a 31-bit unsigned n by a fixed divisor d as one high multiply and a shift:
// with l = ceil(log2 d) and m = floor(2^(31+l) / d) + 1 (which fits 32 bits),
// floor(n / d) = (n * m) >> (31 + l) for every n < 2^31.  d = 1 is flagged by mul = 0.
struct FastDiv {
    uint32_t mul, shift;
};
inline FastDiv make_fast_div(uint32_t d) {
    FastDiv f = {0, 0};
    if (d <= 1) return f;
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    f.mul = (uint32_t)((1ull << (31 + l)) / d + 1);
    f.shift = l - 1;
    return f;
}
__host__ __device__ inline uint32_t fast_div(uint32_t n, FastDiv f) {
#if defined(__HIP_DEVICE_COMPILE__)
    return f.mul ? __umulhi(n, f.mul) >> f.shift : n;
#else
    return f.mul ? (uint32_t)(((unsigned long long)n * f.mul) >> 32) >> f.shift : n;
#endif
}

struct Problem {
    int N, C, H, W, K;
    int TH, TW, T;   // tiles per column / row, total tiles
    int Tp;          // T padded to kTilePad
    int CB;          // ceil(C / 64)
    int Kp;          // K padded to kFilterPad
    FastDiv div_tw, div_th;   // by TW and by TH
};

// tile index t = (n*TH + ty)*TW + tx
__host__ __device__ inline void decode_tile(const Problem& p, int t, int& n, int& ty, int& tx) {
    const uint32_t row = fast_div((uint32_t)t, p.div_tw);   // n*TH + ty
    tx = t - (int)row * p.TW;
    n = (int)fast_div(row, p.div_th);
    ty = (int)row - n * p.TH;
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline size_t round_up(size_t a, size_t b) { return (a + b - 1) / b * b; }

inline Problem make_problem(int N, int C, int H, int W, int K) {
    Problem p;
    p.N = N; p.C = C; p.H = H; p.W = W; p.K = K;
    p.TH = ceil_div(H, 4); p.TW = ceil_div(W, 4);
    p.T = N * p.TH * p.TW;
    p.Tp = ceil_div(p.T, kTilePad) * kTilePad;
    p.CB = ceil_div(C, kCBlock);
    p.Kp = ceil_div(K, kFilterPad) * kFilterPad;
    p.div_tw = make_fast_div((uint32_t)p.TW);
    p.div_th = make_fast_div((uint32_t)p.TH);
    return p;
}

__host__ __device__ inline int num_activation_planes(int mode) { return mode == WG_LOSSLESS ? 138 : 72; }
__host__ __device__ inline int num_filter_planes(int mode) { return mode == WG_LOSSLESS ? 138 : 46; }

// ---- packed filter blob -------------------------------------------------------
// [BlobHeader, 256 B][maxmag: uint32 [Kp][26]][table: ScaleEntry [Kp][26]]
// [operand planes: int8 [CB][Kp/16][planes][16][64]][narrow table, only when C <= 4:
// int16 [Kp][36][4]][limb-pair planes, lossless only: int8 [CB][Kp/8][36][8 filters x 2 limbs][64]],
// each section 256-byte aligned.
// The operand planes are fragment-major: the 1 KB piece (16 filters x 64 channels) that one
// matrix-core instruction consumes is contiguous, and all planes of a (channel block, filter
// block) follow each other, so a kernel steps from plane to plane with constant offsets.
constexpr uint32_t kBlobMagic = 0x33344757u;       // "WG43": signed int8 filters, Winograd-domain values of 12 bits
constexpr uint32_t kBlobMagicInt9 = 0x39344757u;   // "WG49": uint8 filters minus a zero point (int9), values of 13 bits
// Channel limit of the int9 path: 16 y is formed in int32 and |y| <= 9 C 255^2, so 16 * 9 * C * 255^2 < 2^31.
constexpr int kMaxChannelsInt9 = 229;
constexpr uint32_t kBlobVersion = 4;

struct BlobHeader {
    uint32_t magic, version;
    int32_t K, C, mode, range, Kp, CB, planes;
    uint32_t reserved[55];
};
static_assert(sizeof(BlobHeader) == 256, "blob header is one 256-byte block");

struct ScaleEntry {  // per (filter k, free entry): down-scale n/2^p, inverse r/2^q
    int32_t n, p, r, q;
};

constexpr int kFilterFragBytes = 16 * kCBlock;
__host__ __device__ inline size_t filter_plane_offset(int plane, int cb, int k, int c64, int Kp, int nplanes) {
    return ((((size_t)cb * (Kp >> 4) + (k >> 4)) * nplanes + plane) * 16 + (k & 15)) * kCBlock + c64;
}

// Reverse scaling of Section 4.2 for a 32-bit channel sum m: (m * r + 2^(q-1)) >> q with an
// arithmetic shift (q = 0: m * r), r <= 255, q <= 7: one multiply-add with a 64-bit result and
// one funnel shift that takes the 32 bits from bit q on (the result fits 32 bits).  Entries that
// were not scaled carry (r, q) = (1, 0), for which this returns m.
struct ReverseScale {
    int r, q, rnd;
    __device__ inline explicit ReverseScale(const ScaleEntry& se) : ReverseScale(se.r, se.q) {}
    __device__ inline ReverseScale(int r_, int q_) : r(r_), q(q_), rnd(q_ > 0 ? 1 << (q_ - 1) : 0) {}
    __device__ inline int operator()(int m) const {
        const long long t = (long long)m * r + rnd;
        return (int)__builtin_amdgcn_alignbit((uint32_t)(t >> 32), (uint32_t)t, (uint32_t)q);
    }
};

// Layers with at most kNarrowChannels input channels (a network's first layer) are served by a
// kernel that multiplies on the vector ALU; for them the blob also carries the Winograd-domain
// filters (after the scaling, in scaled mode) as 16-bit values, four channel slots per value:
// the 36 real numbers of the 26 free entries in the order 16 real entries, then (Re, Im) of
// each complex entry.
constexpr int kNarrowChannels = 4;
constexpr int kNarrowValues = 36;
constexpr int kNarrowFilterBytes = kNarrowValues * kNarrowChannels * 2;   // 288 per filter

// Lossless blobs also carry every Winograd-domain value as a pair of byte limbs, v = 256 h + l with l the
// low byte of v read as a signed int8 and h = (v + 128) >> 8 in [-8, 8], laid out so that the two limbs of
// a filter are neighbouring ROWS of one matrix-core operand: a 1 KB fragment holds 8 filters x (h, l) x 64
// channels of one value.  Values: the 16 real entries, then (Re, Im) of each of the 10 complex entries.
constexpr int kPairValues = 36;
constexpr int kPairFilters = 8;   // filters per fragment
__host__ __device__ inline size_t filter_pair_offset(int value, int cb, int k, int limb, int c64, int Kp) {
    return (((((size_t)cb * (Kp >> 3) + (k >> 3)) * kPairValues + value) * 16 + 2 * (k & 7) + limb) * kCBlock) + c64;
}

struct BlobLayout {
    size_t maxmag_off, table_off, planes_off, narrow_off, pairs_off, total;
};
inline BlobLayout blob_layout(int Kp, int C, int mode) {
    const int CB = (C + kCBlock - 1) / kCBlock;
    BlobLayout b;
    b.maxmag_off = sizeof(BlobHeader);
    b.table_off = round_up(b.maxmag_off + (size_t)Kp * kEntries * sizeof(uint32_t), 256);
    b.planes_off = round_up(b.table_off + (size_t)Kp * kEntries * sizeof(ScaleEntry), 256);
    b.narrow_off = round_up(b.planes_off + (size_t)num_filter_planes(mode) * CB * Kp * kCBlock, 256);
    b.pairs_off = round_up(b.narrow_off + (C <= kNarrowChannels ? (size_t)Kp * kNarrowFilterBytes : 0), 256);
    b.total = b.pairs_off + (mode == WG_LOSSLESS ? (size_t)kPairValues * CB * Kp * 2 * kCBlock : 0);
    return b;
}

// ---- rational F(2x2,3x3) (Sections 4.1-4.2) ----------------------------------------
// Its packed filter blob: [BlobHeader][maxmag: uint32 [Kp][16]][table: ScaleEntry [Kp][16]]
// [operand planes: int8 [CB][Kp/16][planes][16][64]] with planes = 32 (lossless: entry e as limbs
// 2e, 2e+1) or 16 (scaled).  Tiles are 2x2 outputs: a Problem made by make_problem_f2 counts them.
constexpr int kF2Entries = 16;
constexpr uint32_t kF2BlobMagic = 0x32324757u;  // "WG22"
__host__ __device__ inline int f2_filter_planes(int mode) { return mode == WG_LOSSLESS ? 2 * kF2Entries : kF2Entries; }
struct F2BlobLayout {
    size_t maxmag_off, table_off, planes_off, total;
};
inline F2BlobLayout f2_blob_layout(int Kp, int C, int mode) {
    const int CB = (C + kCBlock - 1) / kCBlock;
    F2BlobLayout b;
    b.maxmag_off = sizeof(BlobHeader);
    b.table_off = round_up(b.maxmag_off + (size_t)Kp * kF2Entries * sizeof(uint32_t), 256);
    b.planes_off = round_up(b.table_off + (size_t)Kp * kF2Entries * sizeof(ScaleEntry), 256);
    b.total = b.planes_off + (size_t)f2_filter_planes(mode) * CB * Kp * kCBlock;
    return b;
}
inline Problem make_problem_f2(int N, int C, int H, int W, int K) {
    Problem p = make_problem(N, C, H, W, K);
    p.TH = ceil_div(H, 2); p.TW = ceil_div(W, 2);
    p.T = N * p.TH * p.TW;
    p.Tp = ceil_div(p.T, kTilePad) * kTilePad;
    p.div_tw = make_fast_div((uint32_t)p.TW);
    p.div_th = make_fast_div((uint32_t)p.TH);
    return p;
}
// is_unsigned: the bytes are uint8 with the given zero point (values = byte - zero_point, the int9
// of Section 4.1); otherwise signed int8 and zero_point is ignored.
hipError_t launch_f2_filter_transform(const int8_t* w, int is_unsigned, int zero_point, int K, int C, int layout, int mode,
                                      void* blob, hipStream_t s);
hipError_t launch_f2_unpack_filter_planes(const void* blob, int8_t* dense, int32_t* table, int K, int C, int mode,
                                          hipStream_t s);
struct Int8Epilogue;   // defined with the single-kernel path's launchers below
hipError_t launch_f2_conv_act_scaled(const int8_t* x, const void* blob, int32_t* y, int32_t* act_table, const Problem& p,
                                     int layout, hipStream_t s);
hipError_t launch_f2_conv(const int8_t* x, int is_unsigned, int zero_point, const void* blob, int32_t* y, const Problem& p,
                          int layout, int mode, const Int8Epilogue& q8, hipStream_t s);

// ---- workspace ------------------------------------------------------------------
// [V: int8 [planes][CB][Tp][64]][M: int32 [46 lossless | 36 scaled][Tp][Kp]]
struct WorkspaceLayout {
    size_t v_off, m_off, total;
};
inline WorkspaceLayout workspace_layout(const Problem& p, int mode) {
    WorkspaceLayout w;
    w.v_off = 0;
    w.m_off = round_up((size_t)num_activation_planes(mode) * p.CB * p.Tp * kCBlock, 256);
    w.total = w.m_off + (size_t)(mode == WG_LOSSLESS ? kMaxWorkspacePlanes : kAccPlanes) * p.Tp * p.Kp * sizeof(int32_t);
    return w;
}

// ---- stage launchers (each enqueues on `s` and returns the launch status) --------
// is_unsigned: the bytes are uint8 with the given zero point (values = byte - zero_point, the int9
// of Section 4.1) and the blob gets kBlobMagicInt9; otherwise signed int8 and zero_point is ignored.
hipError_t launch_filter_transform(const int8_t* w, int is_unsigned, int zero_point, int K, int C, int layout, int mode,
                                   void* blob, hipStream_t s);
hipError_t launch_input_transform(const int8_t* x, const Problem& p, int layout, int mode,
                                  int8_t* V, hipStream_t s);
hipError_t launch_contraction(const int8_t* V, const void* blob, int32_t* M, const Problem& p,
                              int mode, hipStream_t s);
hipError_t launch_output_transform(const int32_t* M, const void* blob, int32_t* y, const Problem& p,
                                   int layout, int mode, hipStream_t s);
// What the single-kernel path does with a finished int32 output.  out == nullptr: store it to y.
// Otherwise y is unused and the kernel stores int8: v = (y + round) >> shift clamped to
// [lo, 127], followed by a 2x2 stride-2 maximum when pool != 0 (H and W even; a 4x4 output tile
// holds whole pooling windows).
struct Int8Epilogue {
    int8_t* out;
    int shift, round, lo, pool;
};
inline Int8Epilogue no_int8_epilogue() { return Int8Epilogue{nullptr, 0, 0, 0, 0}; }
inline Int8Epilogue make_int8_epilogue(int8_t* out, int shift, bool relu, bool pool) {
    return Int8Epilogue{out, shift, shift > 0 ? 1 << (shift - 1) : 0, relu ? 0 : -128, pool ? 1 : 0};
}
// Single-kernel path (no workspace traffic).
hipError_t launch_fused_conv(const int8_t* x, const void* blob, int32_t* y, const Problem& p, int layout,
                             int mode, const Int8Epilogue& q8, hipStream_t s);
// Test hook: n > 0 makes the single-kernel path use its streaming variant wherever the layout
// allows, with n workgroups per filter block; 0 restores the library's own choice.
void set_stream_workgroups(int n);
// Single-kernel path, lossless mode, channels-last with C % 4 == 0: the form whose filter operand carries
// both limbs of eight filters (see lossless_conv.hip).  set_lossless_variant: 0 the library's choice,
// 1 this form wherever the layout allows, 2 never (test hook).
hipError_t launch_lossless_pair_conv(const int8_t* x, const void* blob, int32_t* y, const Problem& p,
                                     const Int8Epilogue& q8, hipStream_t s);
// 0: this form does not apply (layout) or is switched off, 1: applies, the dispatcher decides, 2: forced by the test hook
int lossless_pair_conv_choice(const int8_t* x, const Problem& p, int layout);
void set_lossless_variant(int v);
// Test hook (both modes): 0 the library's choice, 1 the role-specialised kernel with eight product waves (64 filters
// per workgroup) wherever the layout allows (channels-last, C % 4 = 0, K % 4 = 0), 2 never that form.
void set_scaled_variant(int v);
// The same for the streaming kernel's form with eight product waves (0, 1: wherever the layer streams, 2: never).
void set_stream_variant(int v);
// Single-kernel path with the activations scaled per tile as well (WG_SCALED blob of signed int8 filters).
// act_table: null, or int32 [T][26][4] that receives every tile's (n, p, r, q).
hipError_t launch_fused_conv_act_scaled(const int8_t* x, const void* blob, int32_t* y, int32_t* act_table, const Problem& p,
                                        int layout, hipStream_t s);
// Single-kernel path for uint8 activations with a zero point and a kBlobMagicInt9 blob (C <= kMaxChannelsInt9).
hipError_t launch_fused_conv_u8(const uint8_t* x, int zero_point, const void* blob, int32_t* y, const Problem& p, int layout,
                                int mode, hipStream_t s);
// Single-kernel path for channels-last inputs with C <= kNarrowChannels.
hipError_t launch_narrow_conv(const int8_t* x, const void* blob, int32_t* y, const Problem& p, int mode,
                              const Int8Epilogue& q8, hipStream_t s);
hipError_t launch_direct_conv(const int8_t* x, const int8_t* w, int32_t* y, const Problem& p,
                              int layout, hipStream_t s);
hipError_t launch_requant_relu_pool(const int32_t* y, int8_t* out, int N, int K, int H, int W,
                                    int layout, int shift, int relu, int pool, hipStream_t s);
hipError_t launch_unpack_activation_planes(const int8_t* V, int8_t* dense, const Problem& p, int mode,
                                           hipStream_t s);
hipError_t launch_unpack_filter_planes(const void* blob, int8_t* dense, int32_t* table, int K, int C,
                                       int mode, hipStream_t s);
hipError_t launch_unpack_accumulators(const int32_t* M, int32_t* dense, const Problem& p, int mode,
                                      hipStream_t s);

// Raises a kernel's dynamic LDS limit the first time its launcher runs; safe when several host
// threads make that first call together.  Every call returns the status of the one attempt.
struct LdsLimitOnce {
    std::once_flag once;
    hipError_t status = hipSuccess;
    hipError_t set(const void* kernel, int lds_bytes) {
        std::call_once(once, [&] {
            status = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        });
        return status;
    }
};

// True on the device when the blob header matches; kernels that consume a blob
// return without side effects otherwise.
__device__ inline bool blob_matches(const BlobHeader* h, int K, int C, int mode, uint32_t magic = kBlobMagic) {
    return h->magic == magic && h->version == kBlobVersion && h->K == K && h->C == C &&
           h->mode == mode;
}

// The same check in two steps, for kernels that want the header's load in flight while they do other work: the
// first eight dwords in one scalar load, compared later without short-circuit evaluation (which would turn the
// comparison into a chain of dependent loads).
struct BlobHeaderWords {
    uint32_t w[8];
};
__device__ inline BlobHeaderWords read_blob_header(const void* blob) {
    const uint32_t* h = static_cast<const uint32_t*>(__builtin_assume_aligned(blob, 256));
    BlobHeaderWords out;
#pragma unroll
    for (int i = 0; i < 8; ++i) out.w[i] = h[i];
    return out;
}
__device__ inline bool blob_matches(const BlobHeaderWords& h, int K, int C, int mode) {
    static_assert(offsetof(BlobHeader, mode) == 16, "magic, version, K, C, mode are the first five dwords");
    return (h.w[0] == kBlobMagic) & (h.w[1] == kBlobVersion) & ((int)h.w[2] == K) & ((int)h.w[3] == C) & ((int)h.w[4] == mode);
}

}  // namespace wg
