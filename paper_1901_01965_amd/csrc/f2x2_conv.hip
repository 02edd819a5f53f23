// The rational Winograd algorithm F(2x2,3x3) in integer arithmetic, the running example of
// Sections 4.1-4.2 and the variant the paper's evaluation used (Section 4.4): filter transform
// W = G' g G'^T with G' = 2G (the matrix printed in Section 4.1), the filter precision scaling of
// Section 4.2 per output channel and X-Y location (16 factors per filter), and one kernel for
// input transform, Winograd-domain products on the int8 matrix cores and output transform.
//
// All 16 entries are real.  For int8 data the transformed activations need 11 bits and the
// transformed filters 12, so both travel as two int8 limbs v = 64 h + l (l in 0..63); in scaled
// mode the filters are back in int8 and are a single operand.  Per entry the matrix cores form
//   lossless: hh, hl + lh, ll  (value = 4096 hh + 64 mid + ll)      scaled: h w, l w  (64 hw + lw)
// and, unlike in the F(4x4,3x3) kernel, every accumulator of a wave (16 entries x 3) fits its
// registers for the whole kernel: the matrix cores sum over all input channels and the limbs
// are joined, unscaled (Section 4.2, scaled mode) and run through A^T . A once, at the end.
#include <type_traits>
#include <utility>

#include "input_transform_core.h"
#include "wg_internal.h"

namespace wg {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kF2Tiles = 16;      // tiles per workgroup: the rows of the 16x16x64 matrix-core product
constexpr int kF2Filters = 64;    // filters per workgroup: four 16-wide column blocks, one per wave
constexpr int kF2ActPlanes = 2 * kF2Entries;
constexpr int kF2PlaneBytes = kF2Tiles * kCBlock;            // one operand plane of the tile block in LDS
constexpr int kF2LdsBytes = kF2ActPlanes * kF2PlaneBytes;    // 32 KB
constexpr int kF2StageBytes = 24 * 1024;                     // the output staging's share of it

// ---- filter transform -----------------------------------------------------------------------
// W = G' g G'^T in the row-major order of the matrix printed in Section 4.1.
__device__ inline void f2_filter_entries(const int g[9], int w[16]) {
    int u[4][3];   // G' g
    for (int c = 0; c < 3; ++c) {
        const int g0 = g[c], g1 = g[3 + c], g2 = g[6 + c];
        u[0][c] = 2 * g0;
        u[1][c] = g0 + g1 + g2;
        u[2][c] = g0 - g1 + g2;
        u[3][c] = 2 * g2;
    }
    for (int r = 0; r < 4; ++r) {
        w[4 * r + 0] = 2 * u[r][0];
        w[4 * r + 1] = u[r][0] + u[r][1] + u[r][2];
        w[4 * r + 2] = u[r][0] - u[r][1] + u[r][2];
        w[4 * r + 3] = 2 * u[r][2];
    }
}

// Quantised values as the integers the arithmetic works on: signed int8 as they are, or unsigned
// uint8 minus the zero point (the int9 of Section 4.1).
struct Quantisation {
    int is_unsigned, zero_point;
    __device__ inline int value(int8_t raw) const { return is_unsigned ? (int)(uint8_t)raw - zero_point : (int)raw; }
};

__device__ inline void f2_load_filter(const int8_t* w, Quantisation qn, int k, int c, int K, int C, int layout, int g[9]) {
    for (int i = 0; i < 9; ++i)
        g[i] = (k >= K || c >= C) ? 0
                                  : qn.value(layout == WG_NCHW ? w[((size_t)k * C + c) * 9 + i] : w[((size_t)k * 9 + i) * C + c]);
}

__global__ void f2_blob_init_kernel(uint8_t* blob, int K, int C, int mode, int Kp, int CB, size_t maxmag_off) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) {
        BlobHeader* h = reinterpret_cast<BlobHeader*>(blob);
        h->magic = kF2BlobMagic; h->version = kBlobVersion;
        h->K = K; h->C = C; h->mode = mode; h->range = kWeightRange;
        h->Kp = Kp; h->CB = CB; h->planes = f2_filter_planes(mode);
        for (int j = 0; j < 55; ++j) h->reserved[j] = 0;
    }
    if (i < Kp * kF2Entries) reinterpret_cast<uint32_t*>(blob + maxmag_off)[i] = 0;
}

// Step 2 of Section 4.2: the largest magnitude over the input channels at each of a filter's 16
// locations.  One wave per (filter, 64-channel block).
__global__ __launch_bounds__(64) void f2_maxmag_kernel(const int8_t* w, Quantisation qn, int K, int C, int layout,
                                                       uint32_t* maxmag) {
    const int k = blockIdx.x, c = blockIdx.y * 64 + threadIdx.x;
    int g[9], v[16];
    f2_load_filter(w, qn, k, c, K, C, layout, g);
    f2_filter_entries(g, v);
    for (int e = 0; e < kF2Entries; ++e) {
        int m = abs(v[e]);
        for (int off = 32; off > 0; off >>= 1) m = max(m, __shfl_xor(m, off));
        if (threadIdx.x == 0) atomicMax(&maxmag[k * kF2Entries + e], (uint32_t)m);
    }
}

// Steps 3-4 of Section 4.2 and the reciprocal of its last paragraph (same rule as for the
// complex algorithm): largest n/2^p with a 4-bit n that brings the maximum within the range.
__global__ void f2_table_kernel(const uint32_t* maxmag, ScaleEntry* table, int count, int mode) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    ScaleEntry s = {0, 0, 1, 0};
    const int mx = (int)maxmag[i];
    if (mode == WG_SCALED && mx > kWeightRange) {
        const int num = kWeightRange * 128;
        int y = 0;
        while ((mx << (y + 1)) <= num) ++y;
        s.n = (num * 8) / (mx << y);
        s.p = 10 - y;
        for (int q = 7; q >= 0; --q) {
            const int r = ((2 << (s.p + q)) + s.n) / (2 * s.n);
            if (r <= 255) { s.r = r; s.q = q; break; }
        }
    }
    table[i] = s;
}

// One thread per (filter row k < Kp, channel c < 64*CB); padding rows and channels are zeros.
__global__ __launch_bounds__(256) void f2_pack_kernel(const int8_t* w, Quantisation qn, int K, int C, int layout, int mode,
                                                      int Kp, const ScaleEntry* table, int8_t* planes) {
    const int c = blockIdx.x * 64 + (threadIdx.x & 63);
    const int k = blockIdx.y * 4 + (threadIdx.x >> 6);
    if (k >= Kp) return;
    int g[9], v[16];
    f2_load_filter(w, qn, k, c, K, C, layout, g);
    f2_filter_entries(g, v);
    int8_t* base = planes + filter_plane_offset(0, c >> 6, k, c & 63, Kp, f2_filter_planes(mode));
    for (int e = 0; e < kF2Entries; ++e) {
        if (mode == WG_LOSSLESS) {
            base[(size_t)(2 * e) * kFilterFragBytes] = (int8_t)(v[e] >> 6);
            base[(size_t)(2 * e + 1) * kFilterFragBytes] = (int8_t)(v[e] & 63);
        } else {
            const ScaleEntry s = table[(size_t)k * kF2Entries + e];
            const int scaled = s.n ? (v[e] * s.n + (1 << (s.p - 1))) >> s.p : v[e];   // round half up
            base[(size_t)e * kFilterFragBytes] = (int8_t)scaled;
        }
    }
}

__global__ void f2_unpack_kernel(const int8_t* planes, const ScaleEntry* table, int8_t* dense, int32_t* table_out,
                                 int K, int C, int Kp, int nplanes) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t total = (size_t)nplanes * K * C;
    if (i < total) {
        const int c = (int)(i % C), k = (int)((i / C) % K), pl = (int)(i / ((size_t)C * K));
        dense[i] = planes[filter_plane_offset(pl, c >> 6, k, c & 63, Kp, nplanes)];
    }
    if (i < (size_t)K * kF2Entries) {
        const ScaleEntry s = table[i];
        table_out[4 * i + 0] = s.n; table_out[4 * i + 1] = s.p;
        table_out[4 * i + 2] = s.r; table_out[4 * i + 3] = s.q;
    }
}

// ---- convolution kernel -----------------------------------------------------------------------
// LDS operand plane: the 16-byte piece holding channels 16 c16 .. 16 c16 + 15 of tile `tile`
// (rotated by 4 c16, so that 4-byte writes and 16-byte reads both spread over the banks).
__device__ inline int f2_lds_slot(int c16, int tile) { return c16 * 16 + ((tile + 4 * c16) & 15); }

// How activation bytes become the unsigned u = x + bias the transform works on (so that unpacking
// is a zero extension): signed int8: flip the sign bit, bias 128; uint8 with zero point z: the
// byte itself, bias z.  A pixel that does not exist (padding, channels beyond C) is the bias.
struct ActivationBias {
    uint32_t flip;    // XOR mask on the four packed bytes
    uint32_t bytes;   // the bias in each of the four bytes
    int entry11;      // what the bias leaves at entry (1,1) of B^T d B: 4 * bias
};

// The 4x4 input patch of one tile (rows 2ty-1 .. 2ty+2, columns 2tx-1 .. 2tx+2), four
// consecutive channels per pixel packed into a dword.  Addresses are clamped into the image, so no
// load sits behind a branch, and nothing here uses the loaded data (with 4-byte loads): the
// requests travel until f2_bias_patch() turns them into biased values, where pixels outside the
// image and channels beyond C become the bias itself (x = 0).
template <int LAYOUT, bool VEC4>
__device__ inline void f2_request_patch(const int8_t* __restrict__ x, const Problem& p, const ActivationBias& ab, int n, int ty,
                                     int tx, int c0, uint32_t u[4][4]) {
    const int h0 = 2 * ty - 1, w0 = 2 * tx - 1;
    const uint32_t pixel_stride = LAYOUT == WG_NHWC ? (uint32_t)p.C : 1u;
    uint32_t row_off[4], col_off[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        row_off[a] = (uint32_t)min(max(h0 + a, 0), p.H - 1) * (uint32_t)p.W * pixel_stride;
        col_off[a] = (uint32_t)min(max(w0 + a, 0), p.W - 1) * pixel_stride;
    }
    const int8_t* img = x + (size_t)n * p.C * p.H * p.W;
    if constexpr (VEC4) {
        const int8_t* src = img + (c0 < p.C ? c0 : 0);
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) u[a][b] = *reinterpret_cast<const uint32_t*>(src + (row_off[a] + col_off[b]));
    } else {
        const uint32_t cstride = LAYOUT == WG_NHWC ? 1u : (uint32_t)p.H * (uint32_t)p.W;
        uint32_t chan_off[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) chan_off[i] = (uint32_t)min(c0 + i, p.C - 1) * cstride;
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                uint32_t word = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t e = (uint8_t)img[row_off[a] + col_off[b] + chan_off[i]];
                    word |= (c0 + i < p.C ? e : ((ab.bytes ^ ab.flip) & 0xffu)) << (8 * i);   // beyond C: x = 0
                }
                u[a][b] = word;
            }
    }
}

__device__ inline void f2_bias_patch(const Problem& p, const ActivationBias& ab, int ty, int tx, int c0, uint32_t u[4][4]) {
    const int h0 = 2 * ty - 1, w0 = 2 * tx - 1;
    const bool have = c0 < p.C;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const bool inside = have && (unsigned)(h0 + a) < (unsigned)p.H && (unsigned)(w0 + b) < (unsigned)p.W;
            u[a][b] = inside ? (u[a][b] ^ ab.flip) : ab.bytes;
        }
}

// The 1-D rule of B^T for F(2,3): t0 = v0 - v2, t1 = v1 + v2, t2 = v2 - v1, t3 = v1 - v3.
__device__ inline void f2_bt_rule(Quad v0, Quad v1, Quad v2, Quad v3, Quad t[4]) {
    t[0] = v0 - v2;
    t[1] = v1 + v2;
    t[2] = v2 - v1;
    t[3] = v1 - v3;
}

// D = B^T d B of one patch (four channels), entry e = 4 r + c.  A constant patch transforms to
// zero everywhere except entry (1,1), where the four +1 coefficients add up: the bias leaves
// 4 * bias there and is removed by one subtraction.
__device__ inline void f2_patch_entries(const uint32_t u[4][4], int entry11, Quad d[kF2Entries]) {
    Quad col[4][4];   // col[b][r]: row r of B^T d, column b
#pragma unroll
    for (int b = 0; b < 4; ++b)
        f2_bt_rule(unpack_u8x4(u[0][b]), unpack_u8x4(u[1][b]), unpack_u8x4(u[2][b]), unpack_u8x4(u[3][b]), col[b]);
    const s16x2 bias11 = {(short)entry11, (short)entry11};
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        f2_bt_rule(col[0][r], col[1][r], col[2][r], col[3][r], d + 4 * r);
        if (r == 1) d[5] = Quad{d[5].a - bias11, d[5].b - bias11};
    }
}

// Entry e as two limbs: planes 2e (high) and 2e + 1 (low).
__device__ inline void f2_transform_patch(const uint32_t u[4][4], int entry11, int8_t* lds_piece) {
    Quad d[kF2Entries];
    f2_patch_entries(u, entry11, d);
#pragma unroll
    for (int e = 0; e < kF2Entries; ++e) {
        const Quad hi = Quad{d[e].a >> 6, d[e].b >> 6};
        *reinterpret_cast<uint32_t*>(lds_piece + (2 * e) * kF2PlaneBytes) = pack_low_bytes(hi);
        *reinterpret_cast<uint32_t*>(lds_piece + (2 * e + 1) * kF2PlaneBytes) = pack_low_bytes(d[e]) & 0x3f3f3f3fu;
    }
}

template <class F, int... Is>
__device__ inline void f2_static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ inline void f2_static_for(F&& f) {
    f2_static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// With eight or more filter blocks, workgroups are dealt to the eight XCDs (round-robin in
// launch order) so that all tile blocks of a filter block share one L2.
__device__ inline void f2_block_coordinates(int& bx, int& by) {
    bx = blockIdx.x;
    by = blockIdx.y;
    const int total = gridDim.x * gridDim.y;
    if (gridDim.y >= 8 && (total & 7) == 0) {
        const int launch = blockIdx.y * gridDim.x + blockIdx.x;
        const int w = (launch & 7) * (total >> 3) + (launch >> 3);
        by = w / (int)gridDim.x;
        bx = w - by * (int)gridDim.x;
    }
}

// Where a workgroup's tiles and filters sit, as every phase of the kernels below needs it.
struct F2Block {
    int tid, lane, wave;
    int tile0, kbase, k;          // first tile, first filter, this lane's filter (< Kp)
    int my_n, my_ty, my_tx;       // coordinates of tile tile0 + (lane & 15)
};

// Y = A^T M A with A^T = [1 1 1 0; 0 1 -1 -1]: rows first, then columns; the rescale by 2^-2
// undoes G' = 2G on both sides (rnd = 0: exact, lossless mode; rnd = 2: round half up).  Register
// q of m[e] belongs to tile 4 (lane / 16) + q and filter k.  The operand planes in LDS must be
// dead for all waves' products when this is called (it synchronises before it overwrites them).
// Q8: instead of the int32 store, v = (y + round) >> shift clamped to [lo, 127] goes to q8.out as
// int8; with q8.pool the tile's four outputs (one 2x2 pooling window) are reduced to their maximum.
__device__ inline v4i f2_requantise(v4i v, const Int8Epilogue& q) {
    v = (v + q.round) >> q.shift;
    const v4i lo = {q.lo, q.lo, q.lo, q.lo}, hi = {127, 127, 127, 127};
    return __builtin_elementwise_min(__builtin_elementwise_max(v, lo), hi);
}
template <int LAYOUT, bool Q8 = false>
__device__ __forceinline__ void f2_output_transform_store(const v4i (&m)[kF2Entries], int rnd, const F2Block& b,
                                                          const Problem& p, int8_t* lds, int32_t* __restrict__ y,
                                                          const Int8Epilogue& q8 = Int8Epilogue{nullptr, 0, 0, 0, 0}) {
    const int lane = b.lane;
    v4i z[2][4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        z[0][c] = m[c] + m[4 + c] + m[8 + c];
        z[1][c] = m[4 + c] - m[8 + c] - m[12 + c];
    }
    v4i out[4];   // output pixel 2 i + j
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        out[2 * i + 0] = (z[i][0] + z[i][1] + z[i][2] + rnd) >> 2;
        out[2 * i + 1] = (z[i][1] - z[i][2] - z[i][3] + rnd) >> 2;
    }
    // int8 epilogue: NO outputs per tile (one after pooling), on a grid of Ho x Wo pixels
    const bool pooled = Q8 && q8.pool != 0;
    const int NO = pooled ? 1 : 4, Ho = pooled ? p.H >> 1 : p.H, Wo = pooled ? p.W >> 1 : p.W;
    if constexpr (Q8) {
#pragma unroll
        for (int o = 0; o < 4; ++o) out[o] = f2_requantise(out[o], q8);
        if (pooled)
            out[0] = __builtin_elementwise_max(__builtin_elementwise_max(out[0], out[1]), __builtin_elementwise_max(out[2], out[3]));
    }
    if (LAYOUT == WG_NHWC && (p.K & 3) == 0) {
        // Channels-last with K a multiple of four: staged filter-fastest, stage[pixel][tile][68]
        // (64 filters, rows padded to 68 dwords), then a thread stores four consecutive filters
        // and sixteen lanes cover the 256 contiguous bytes this block owns of a pixel.
        constexpr int kRow = 68;
        static_assert(4 * 16 * kRow * 4 <= kF2StageBytes, "staging fits its share of the LDS");
        __syncthreads();   // the operand planes are dead
        int* stage = reinterpret_cast<int*>(lds);
#pragma unroll
        for (int o = 0; o < 4; ++o)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (o < NO) stage[(o * 16 + 4 * (lane >> 4) + q) * kRow + b.wave * 16 + (lane & 15)] = out[o][q];
        __syncthreads();
        const int k4 = b.tid & 15, tile = b.tid >> 4;   // thread: filters 4 k4 .. 4 k4 + 3 of tile `tile`, all four pixels
        const int n = __shfl(b.my_n, tile), ty = __shfl(b.my_ty, tile), tx = __shfl(b.my_tx, tile);
        const int kk = b.kbase + 4 * k4;
        if (b.tile0 + tile < p.T && kk < p.K) {
#pragma unroll
            for (int o = 0; o < 4; ++o) {
                if (o >= NO) break;
                const int h = pooled ? ty : 2 * ty + (o >> 1), w = pooled ? tx : 2 * tx + (o & 1);
                if (h >= Ho || w >= Wo) continue;
                const v4i v = *reinterpret_cast<const v4i*>(stage + (o * 16 + tile) * kRow + 4 * k4);
                const size_t at = (((size_t)n * Ho + h) * Wo + w) * p.K + kk;
                if constexpr (Q8)
                    *reinterpret_cast<uint32_t*>(q8.out + at) = (uint32_t)(v[0] & 0xff) | ((uint32_t)(v[1] & 0xff) << 8) |
                                                                ((uint32_t)(v[2] & 0xff) << 16) | ((uint32_t)v[3] << 24);
                else
                    *reinterpret_cast<v4i*>(y + at) = v;
            }
        }
        return;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int tl = 4 * (lane >> 4) + q;
        const int n = __shfl(b.my_n, tl), ty = __shfl(b.my_ty, tl), tx = __shfl(b.my_tx, tl);   // all lanes take part
        if (b.tile0 + tl >= p.T || b.k >= p.K) continue;
#pragma unroll
        for (int o = 0; o < 4; ++o) {
            if (o >= NO) break;
            const int h = pooled ? ty : 2 * ty + (o >> 1), w = pooled ? tx : 2 * tx + (o & 1);
            if (h >= Ho || w >= Wo) continue;
            const size_t at = LAYOUT == WG_NHWC ? (((size_t)n * Ho + h) * Wo + w) * p.K + b.k
                                                : (((size_t)n * p.K + b.k) * Ho + h) * Wo + w;
            if constexpr (Q8) q8.out[at] = (int8_t)out[o][q];
            else              y[at] = out[o][q];
        }
    }
}

// grid: (ceil(T/16), Kp/64), 256 threads.  Transform phase: thread = (tile, four channels).
// Product phase: wave w owns filter block w (16 filters) of the 16 tiles for all 16 entries; the
// filter fragments travel through a ring that is filled before the transform, the activation
// fragments of entry e + 2 are read from LDS while entry e multiplies.
template <int LAYOUT, bool VEC4, int MODE, bool Q8>
__global__ __launch_bounds__(256) void f2_conv_kernel(const int8_t* __restrict__ x, const uint8_t* __restrict__ blob,
                                                      size_t table_off, size_t planes_off, int32_t* __restrict__ y,
                                                      Problem p, ActivationBias ab, Int8Epilogue q8) {
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int bx, by;
    f2_block_coordinates(bx, by);
    const int tile0 = bx * kF2Tiles;
    const int kbase = by * kF2Filters;
    const int k = kbase + wave * 16 + (lane & 15);   // this lane's filter (< Kp)
    const BlobHeader* hdr = reinterpret_cast<const BlobHeader*>(blob);
    if (!(hdr->magic == kF2BlobMagic && hdr->version == kBlobVersion && hdr->K == p.K && hdr->C == p.C && hdr->mode == MODE))
        return;

    constexpr int NA = MODE == WG_LOSSLESS ? 3 : 2;          // accumulators per entry
    constexpr int NBP = MODE == WG_LOSSLESS ? 2 : 1;         // filter planes per entry
    constexpr int NP = MODE == WG_LOSSLESS ? 2 * kF2Entries : kF2Entries;
    v4i acc[kF2Entries][NA];
#pragma unroll
    for (int e = 0; e < kF2Entries; ++e)
#pragma unroll
        for (int i = 0; i < NA; ++i) acc[e][i] = (v4i){0, 0, 0, 0};

    // every lane decodes tile (lane & 15) of the block once; the transform phase fetches the
    // coordinates of its own tile (tid / 16) from that lane
    int my_n = 0, my_ty = 0, my_tx = 0;
    if (tile0 + (lane & 15) < p.T) decode_tile(p, tile0 + (lane & 15), my_n, my_ty, my_tx);
    const int a_tile = tid >> 4, cq = tid & 15;
    const int a_n = __shfl(my_n, a_tile), a_ty = __shfl(my_ty, a_tile), a_tx = __shfl(my_tx, a_tile);
    int8_t* put = lds + f2_lds_slot(cq >> 2, a_tile) * 16 + (cq & 3) * 4;
    const int8_t* a_lds = lds + f2_lds_slot(lane >> 4, lane & 15) * 16;
    const int8_t* b_lane = reinterpret_cast<const int8_t*>(blob + planes_off) +
                           filter_plane_offset(0, 0, k, (lane >> 4) * 16, p.Kp, NP);
    const size_t b_block_stride = (size_t)(p.Kp >> 4) * NP * kFilterFragBytes;

    // Workgroups that run side by side on an XCD read the same filter fragments; each starts at a
    // channel block of its own (the integer sums do not depend on the order) so that they do not
    // all ask the same L2 channels for the same lines at the same time.
    int cb = bx % p.CB;
    uint32_t u[4][4];
    f2_request_patch<LAYOUT, VEC4>(x, p, ab, a_n, a_ty, a_tx, cb * kCBlock + 4 * cq, u);
    // filter fragments in flight: requested before the transform, they arrive under it
    constexpr int kRing = MODE == WG_LOSSLESS ? 4 : 6;
    for (int step = 0; step < p.CB; ++step) {
        const int8_t* b_cb = b_lane + cb * b_block_stride;
        v4i bf[kRing][NBP], af[3][2];
        auto request_b = [&](auto E) {
            constexpr int e = E;
#pragma unroll
            for (int i = 0; i < NBP; ++i)
                bf[e % kRing][i] = *reinterpret_cast<const v4i*>(b_cb + (NBP * e + i) * kFilterFragBytes);
        };
        auto request_a = [&](auto E) {
            constexpr int e = E;
            af[e % 3][0] = *reinterpret_cast<const v4i*>(a_lds + (2 * e) * kF2PlaneBytes);
            af[e % 3][1] = *reinterpret_cast<const v4i*>(a_lds + (2 * e + 1) * kF2PlaneBytes);
        };
        f2_static_for<kRing - 1>([&](auto E) { request_b(E); });
        __builtin_amdgcn_sched_barrier(0);
        if (step > 0) __syncthreads();   // the previous block's operand planes have been consumed
        f2_bias_patch(p, ab, a_ty, a_tx, cb * kCBlock + 4 * cq, u);
        f2_transform_patch(u, ab.entry11, put);
        cb = cb + 1 == p.CB ? 0 : cb + 1;
        // the next channel block's patch travels while this one multiplies
        if (step + 1 < p.CB) f2_request_patch<LAYOUT, VEC4>(x, p, ab, a_n, a_ty, a_tx, cb * kCBlock + 4 * cq, u);
        __syncthreads();               // the operand planes are complete
        request_a(std::integral_constant<int, 0>{});
        request_a(std::integral_constant<int, 1>{});
        f2_static_for<kF2Entries>([&](auto E) {
            constexpr int e = E;
            if constexpr (e + kRing - 1 < kF2Entries) request_b(std::integral_constant<int, e + kRing - 1>{});
            if constexpr (e + 2 < kF2Entries) request_a(std::integral_constant<int, e + 2>{});
            const v4i ah = af[e % 3][0], al = af[e % 3][1];
            if constexpr (MODE == WG_LOSSLESS) {
                acc[e][0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ah, bf[e % kRing][0], acc[e][0], 0, 0, 0);
                acc[e][1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ah, bf[e % kRing][1], acc[e][1], 0, 0, 0);
                acc[e][2] = __builtin_amdgcn_mfma_i32_16x16x64_i8(al, bf[e % kRing][1], acc[e][2], 0, 0, 0);
                acc[e][1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(al, bf[e % kRing][0], acc[e][1], 0, 0, 0);
            } else {
                acc[e][0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ah, bf[e % kRing][0], acc[e][0], 0, 0, 0);
                acc[e][1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(al, bf[e % kRing][0], acc[e][1], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    }

    // ---- join the limbs, undo the filter scaling, output transform --------------------------
    v4i m[kF2Entries];
#pragma unroll
    for (int e = 0; e < kF2Entries; ++e) {
        if constexpr (MODE == WG_LOSSLESS) {
            m[e] = (((acc[e][0] << 6) + acc[e][1]) << 6) + acc[e][2];
        } else {
            m[e] = (acc[e][0] << 6) + acc[e][1];
            const ReverseScale unscale(reinterpret_cast<const ScaleEntry*>(blob + table_off)[(size_t)k * kF2Entries + e]);
#pragma unroll
            for (int q = 0; q < 4; ++q) m[e][q] = unscale(m[e][q]);
        }
    }
    const F2Block blk = {tid, lane, wave, tile0, kbase, k, my_n, my_ty, my_tx};
    f2_output_transform_store<LAYOUT, Q8>(m, MODE == WG_SCALED ? 2 : 0, blk, p, lds, y, q8);
}

// ---- activations scaled as well -------------------------------------------------------------------
// Section 4.1 closes with the remark that the analysis of Section 4.2 applies to B^T d B too
// (11 bits for int8 data).  The rule here is that section's with a tile in the place of an output
// feature map: the largest magnitude over the input channels at each of a tile's 16 X-Y locations
// decides one factor n/2^p, every channel's value there is multiplied by it (round half up), and
// the channel sums are multiplied back by its reciprocal r/2^q after the filter's.  Both operands
// are then single int8 values: one matrix-core instruction per entry and channel block.
//
// (n, p, r, q) for every possible maximum of int8 data, one byte each (n = 0: within the range,
// nothing applied).
constexpr int kF2ActMax = 4 * 128;
struct F2ActScaleTable {
    uint32_t v[kF2ActMax + 1];
};
constexpr F2ActScaleTable f2_make_act_scale_table() {
    F2ActScaleTable t = {};
    for (int mx = 0; mx <= kF2ActMax; ++mx) {
        uint32_t n = 0, p = 0, r = 1, q = 0;
        if (mx > kWeightRange) {
            const int num = kWeightRange * 128;
            int y = 0;
            while ((mx << (y + 1)) <= num) ++y;
            n = (uint32_t)((num * 8) / (mx << y));
            p = (uint32_t)(10 - y);
            for (int qq = 7; qq >= 0; --qq) {
                const uint32_t rr = ((2u << (p + qq)) + n) / (2 * n);
                if (rr <= 255) { r = rr; q = (uint32_t)qq; break; }
            }
        }
        t.v[mx] = n | (p << 8) | (r << 16) | (q << 24);
    }
    return t;
}
__device__ const F2ActScaleTable kF2ActScale = f2_make_act_scale_table();

constexpr int kF2NpOff = 28 * 1024;   // LDS: packed table entries [tile][entry], read by the transform threads
constexpr int kF2RqOff = 29 * 1024;   // the same entries [entry][tile], read by the finishing lanes
static_assert(kF2StageBytes <= kF2NpOff && kF2RqOff + 1024 <= kF2LdsBytes, "LDS regions");

// grid and roles as in f2_conv_kernel; the blob is a WG_SCALED one.  Pass 1 transforms every
// channel block of the workgroup's 16 tiles and keeps the running maxima; the 256 threads then
// look up one (tile, location) each; pass 2 transforms again (the patches now come from the
// caches), scales, and multiplies.  act_table (may be null) receives int32 [T][16][4] = (n,p,r,q).
template <int LAYOUT, bool VEC4>
__global__ __launch_bounds__(256) void f2_conv_act_scaled_kernel(const int8_t* __restrict__ x,
                                                                 const uint8_t* __restrict__ blob, size_t table_off,
                                                                 size_t planes_off, int32_t* __restrict__ y,
                                                                 int32_t* __restrict__ act_table, Problem p,
                                                                 ActivationBias ab) {
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int bx, by;
    f2_block_coordinates(bx, by);
    const int tile0 = bx * kF2Tiles;
    const int kbase = by * kF2Filters;
    const int k = kbase + wave * 16 + (lane & 15);
    const BlobHeader* hdr = reinterpret_cast<const BlobHeader*>(blob);
    if (!(hdr->magic == kF2BlobMagic && hdr->version == kBlobVersion && hdr->K == p.K && hdr->C == p.C &&
          hdr->mode == WG_SCALED))
        return;

    int my_n = 0, my_ty = 0, my_tx = 0;
    if (tile0 + (lane & 15) < p.T) decode_tile(p, tile0 + (lane & 15), my_n, my_ty, my_tx);
    const int a_tile = tid >> 4, cq = tid & 15;
    const int a_n = __shfl(my_n, a_tile), a_ty = __shfl(my_ty, a_tile), a_tx = __shfl(my_tx, a_tile);
    uint32_t* np_tab = reinterpret_cast<uint32_t*>(lds + kF2NpOff);
    uint32_t* rq_tab = reinterpret_cast<uint32_t*>(lds + kF2RqOff);

    // ---- pass 1: largest magnitude per (tile, location) over all channels ------------------------
    const int first_cb = bx % p.CB;   // see f2_conv_kernel: neighbours start at different channel blocks
    int cb = first_cb;
    uint32_t u[4][4];
    f2_request_patch<LAYOUT, VEC4>(x, p, ab, a_n, a_ty, a_tx, cb * kCBlock + 4 * cq, u);
    s16x2 mx[kF2Entries];
#pragma unroll
    for (int e = 0; e < kF2Entries; ++e) mx[e] = (s16x2){0, 0};
    for (int step = 0; step < p.CB; ++step) {
        Quad d[kF2Entries];
        f2_bias_patch(p, ab, a_ty, a_tx, cb * kCBlock + 4 * cq, u);
        f2_patch_entries(u, ab.entry11, d);
        cb = cb + 1 == p.CB ? 0 : cb + 1;
        if (step + 1 < p.CB) f2_request_patch<LAYOUT, VEC4>(x, p, ab, a_n, a_ty, a_tx, cb * kCBlock + 4 * cq, u);
#pragma unroll
        for (int e = 0; e < kF2Entries; ++e) {
            const s16x2 zero = {0, 0};
            const s16x2 ma = __builtin_elementwise_max(d[e].a, zero - d[e].a);
            const s16x2 mb = __builtin_elementwise_max(d[e].b, zero - d[e].b);
            mx[e] = __builtin_elementwise_max(mx[e], __builtin_elementwise_max(ma, mb));
        }
    }
    // the first patch of pass 2 travels during the reduction
    cb = first_cb;
    f2_request_patch<LAYOUT, VEC4>(x, p, ab, a_n, a_ty, a_tx, cb * kCBlock + 4 * cq, u);
    // over the sixteen threads of a tile (consecutive lanes), two locations per register
    s16x2 pm[kF2Entries / 2];
#pragma unroll
    for (int j = 0; j < kF2Entries / 2; ++j) {
        pm[j] = (s16x2){max(mx[2 * j].x, mx[2 * j].y), max(mx[2 * j + 1].x, mx[2 * j + 1].y)};
#pragma unroll
        for (int off = 1; off < 16; off <<= 1)
            pm[j] = __builtin_elementwise_max(pm[j], as_s16x2((uint32_t)__shfl_xor((int)as_u32(pm[j]), off)));
    }
    {   // thread (tile, cq) looks up location cq of its tile
        int mine = 0;
#pragma unroll
        for (int e = 0; e < kF2Entries; ++e)
            if (cq == e) mine = (e & 1) ? pm[e / 2].y : pm[e / 2].x;
        const uint32_t entry = kF2ActScale.v[min(mine, kF2ActMax)];
        np_tab[a_tile * 16 + cq] = entry;
        rq_tab[cq * 16 + a_tile] = entry;
        if (act_table != nullptr && by == 0 && tile0 + a_tile < p.T)
            *reinterpret_cast<v4i*>(act_table + ((size_t)(tile0 + a_tile) * kF2Entries + cq) * 4) =
                (v4i){(int)(entry & 255u), (int)((entry >> 8) & 255u), (int)((entry >> 16) & 255u), (int)(entry >> 24)};
    }
    __syncthreads();
    s16x2 mul[kF2Entries], shift[kF2Entries], half[kF2Entries];
#pragma unroll
    for (int e = 0; e < kF2Entries; ++e) {
        const uint32_t t = np_tab[a_tile * 16 + e];
        const short n = (short)max((int)(t & 255u), 1), sh = (short)((t >> 8) & 255u);
        const short h = (short)((1 << sh) >> 1);
        mul[e] = (s16x2){n, n};
        shift[e] = (s16x2){sh, sh};
        half[e] = (s16x2){h, h};
    }

    // ---- pass 2: scaled operands, products ----------------------------------------------------------
    v4i acc[kF2Entries];
#pragma unroll
    for (int e = 0; e < kF2Entries; ++e) acc[e] = (v4i){0, 0, 0, 0};
    int8_t* put = lds + f2_lds_slot(cq >> 2, a_tile) * 16 + (cq & 3) * 4;
    const int8_t* a_lds = lds + f2_lds_slot(lane >> 4, lane & 15) * 16;
    const int8_t* b_lane = reinterpret_cast<const int8_t*>(blob + planes_off) +
                           filter_plane_offset(0, 0, k, (lane >> 4) * 16, p.Kp, kF2Entries);
    const size_t b_block_stride = (size_t)(p.Kp >> 4) * kF2Entries * kFilterFragBytes;
    constexpr int kRing = 8;   // filter fragments in flight: requested before the transform, they arrive under it
    for (int step = 0; step < p.CB; ++step) {
        const int8_t* b_cb = b_lane + cb * b_block_stride;
        const int c0 = cb * kCBlock + 4 * cq;
        cb = cb + 1 == p.CB ? 0 : cb + 1;
        v4i bf[kRing], af[3];
        auto request_b = [&](auto E) {
            constexpr int e = E;
            bf[e % kRing] = *reinterpret_cast<const v4i*>(b_cb + e * kFilterFragBytes);
        };
        auto request_a = [&](auto E) {
            constexpr int e = E;
            af[e % 3] = *reinterpret_cast<const v4i*>(a_lds + e * kF2PlaneBytes);
        };
        f2_static_for<kRing - 1>([&](auto E) { request_b(E); });
        __builtin_amdgcn_sched_barrier(0);
        if (step > 0) __syncthreads();   // the previous block's operand planes have been consumed
        {
            Quad d[kF2Entries];
            f2_bias_patch(p, ab, a_ty, a_tx, c0, u);
            f2_patch_entries(u, ab.entry11, d);
#pragma unroll
            for (int e = 0; e < kF2Entries; ++e) {
                const Quad v = Quad{(d[e].a * mul[e] + half[e]) >> shift[e], (d[e].b * mul[e] + half[e]) >> shift[e]};
                *reinterpret_cast<uint32_t*>(put + e * kF2PlaneBytes) = pack_low_bytes(v);
            }
        }
        if (step + 1 < p.CB) f2_request_patch<LAYOUT, VEC4>(x, p, ab, a_n, a_ty, a_tx, cb * kCBlock + 4 * cq, u);
        __syncthreads();               // the operand planes are complete
        request_a(std::integral_constant<int, 0>{});
        request_a(std::integral_constant<int, 1>{});
        f2_static_for<kF2Entries>([&](auto E) {
            constexpr int e = E;
            if constexpr (e + kRing - 1 < kF2Entries) request_b(std::integral_constant<int, e + kRing - 1>{});
            if constexpr (e + 2 < kF2Entries) request_a(std::integral_constant<int, e + 2>{});
            acc[e] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[e % 3], bf[e % kRing], acc[e], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        });
    }

    // ---- undo the filter's factor, then the tile's; output transform ---------------------------------
#pragma unroll
    for (int e = 0; e < kF2Entries; ++e) {
        const ReverseScale filter_side(reinterpret_cast<const ScaleEntry*>(blob + table_off)[(size_t)k * kF2Entries + e]);
        const v4i rq = *reinterpret_cast<const v4i*>(rq_tab + e * 16 + 4 * (lane >> 4));
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const ReverseScale tile_side((int)(((uint32_t)rq[q] >> 16) & 255u), (int)((uint32_t)rq[q] >> 24));
            acc[e][q] = tile_side(filter_side(acc[e][q]));
        }
    }
    const F2Block blk = {tid, lane, wave, tile0, kbase, k, my_n, my_ty, my_tx};
    f2_output_transform_store<LAYOUT>(acc, 2, blk, p, lds, y);
}


template <int LAYOUT, bool VEC4, int MODE, bool Q8>
hipError_t launch(const int8_t* x, const uint8_t* blob, const F2BlobLayout& bl, int32_t* y, const Problem& p,
                  const ActivationBias& ab, const Int8Epilogue& q8, hipStream_t s) {
    static LdsLimitOnce lds_limit;   // per template instance
    if (hipError_t e = lds_limit.set(reinterpret_cast<const void*>(&f2_conv_kernel<LAYOUT, VEC4, MODE, Q8>), kF2LdsBytes)) return e;
    dim3 grid(ceil_div(p.T, kF2Tiles), p.Kp / kF2Filters);
    f2_conv_kernel<LAYOUT, VEC4, MODE, Q8><<<grid, 256, kF2LdsBytes, s>>>(x, blob, bl.table_off, bl.planes_off, y, p, ab, q8);
    return hipGetLastError();
}

template <int LAYOUT, bool VEC4>
hipError_t launch_mode(const int8_t* x, const uint8_t* blob, const F2BlobLayout& bl, int32_t* y, const Problem& p, int mode,
                       const ActivationBias& ab, const Int8Epilogue& q8, hipStream_t s) {
    if (q8.out != nullptr)
        return mode == WG_LOSSLESS ? launch<LAYOUT, VEC4, WG_LOSSLESS, true>(x, blob, bl, y, p, ab, q8, s)
                                   : launch<LAYOUT, VEC4, WG_SCALED, true>(x, blob, bl, y, p, ab, q8, s);
    return mode == WG_LOSSLESS ? launch<LAYOUT, VEC4, WG_LOSSLESS, false>(x, blob, bl, y, p, ab, q8, s)
                               : launch<LAYOUT, VEC4, WG_SCALED, false>(x, blob, bl, y, p, ab, q8, s);
}

template <int LAYOUT, bool VEC4>
hipError_t launch_act_scaled(const int8_t* x, const uint8_t* blob, const F2BlobLayout& bl, int32_t* y, int32_t* act_table,
                             const Problem& p, const ActivationBias& ab, hipStream_t s) {
    static LdsLimitOnce lds_limit;   // per template instance
    if (hipError_t e = lds_limit.set(reinterpret_cast<const void*>(&f2_conv_act_scaled_kernel<LAYOUT, VEC4>), kF2LdsBytes)) return e;
    dim3 grid(ceil_div(p.T, kF2Tiles), p.Kp / kF2Filters);
    f2_conv_act_scaled_kernel<LAYOUT, VEC4><<<grid, 256, kF2LdsBytes, s>>>(x, blob, bl.table_off, bl.planes_off, y, act_table,
                                                                          p, ab);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_f2_filter_transform(const int8_t* w, int is_unsigned, int zero_point, int K, int C, int layout, int mode,
                                      void* blob_v, hipStream_t s) {
    const Quantisation qn = {is_unsigned, zero_point};
    uint8_t* blob = static_cast<uint8_t*>(blob_v);
    const int Kp = ceil_div(K, kFilterPad) * kFilterPad, CB = ceil_div(C, kCBlock);
    const F2BlobLayout bl = f2_blob_layout(Kp, C, mode);
    uint32_t* maxmag = reinterpret_cast<uint32_t*>(blob + bl.maxmag_off);
    ScaleEntry* table = reinterpret_cast<ScaleEntry*>(blob + bl.table_off);
    const int entries = Kp * kF2Entries;
    f2_blob_init_kernel<<<ceil_div(entries, 256), 256, 0, s>>>(blob, K, C, mode, Kp, CB, bl.maxmag_off);
    if (mode == WG_SCALED) f2_maxmag_kernel<<<dim3(K, CB), 64, 0, s>>>(w, qn, K, C, layout, maxmag);
    f2_table_kernel<<<ceil_div(entries, 256), 256, 0, s>>>(maxmag, table, entries, mode);
    f2_pack_kernel<<<dim3(CB, ceil_div(Kp, 4)), 256, 0, s>>>(w, qn, K, C, layout, mode, Kp, table,
                                                             reinterpret_cast<int8_t*>(blob + bl.planes_off));
    return hipGetLastError();
}

hipError_t launch_f2_unpack_filter_planes(const void* blob_v, int8_t* dense, int32_t* table_out, int K, int C, int mode,
                                          hipStream_t s) {
    const uint8_t* blob = static_cast<const uint8_t*>(blob_v);
    const int Kp = ceil_div(K, kFilterPad) * kFilterPad;
    const F2BlobLayout bl = f2_blob_layout(Kp, C, mode);
    const int nplanes = f2_filter_planes(mode);
    const size_t total = (size_t)nplanes * K * C;
    const size_t threads = total > (size_t)K * kF2Entries ? total : (size_t)K * kF2Entries;
    f2_unpack_kernel<<<(unsigned)((threads + 255) / 256), 256, 0, s>>>(
        reinterpret_cast<const int8_t*>(blob + bl.planes_off), reinterpret_cast<const ScaleEntry*>(blob + bl.table_off), dense,
        table_out, K, C, Kp, nplanes);
    return hipGetLastError();
}

hipError_t launch_f2_conv(const int8_t* x, int is_unsigned, int zero_point, const void* blob, int32_t* y, const Problem& p,
                          int layout, int mode, const Int8Epilogue& q8, hipStream_t s) {
    const uint32_t bias = is_unsigned ? (uint32_t)zero_point : 128u;
    const ActivationBias ab = {is_unsigned ? 0u : 0x80808080u, bias * 0x01010101u, (int)(4 * bias)};
    const F2BlobLayout bl = f2_blob_layout(p.Kp, p.C, mode);
    const uint8_t* b = static_cast<const uint8_t*>(blob);
    if (layout == WG_NHWC && p.C % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 4 == 0)
        return launch_mode<WG_NHWC, true>(x, b, bl, y, p, mode, ab, q8, s);
    if (layout == WG_NHWC) return launch_mode<WG_NHWC, false>(x, b, bl, y, p, mode, ab, q8, s);
    return launch_mode<WG_NCHW, false>(x, b, bl, y, p, mode, ab, q8, s);
}

hipError_t launch_f2_conv_act_scaled(const int8_t* x, const void* blob, int32_t* y, int32_t* act_table, const Problem& p,
                                     int layout, hipStream_t s) {
    const ActivationBias ab = {0x80808080u, 128u * 0x01010101u, 4 * 128};
    const F2BlobLayout bl = f2_blob_layout(p.Kp, p.C, WG_SCALED);
    const uint8_t* b = static_cast<const uint8_t*>(blob);
    if (layout == WG_NHWC && p.C % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 4 == 0)
        return launch_act_scaled<WG_NHWC, true>(x, b, bl, y, act_table, p, ab, s);
    if (layout == WG_NHWC) return launch_act_scaled<WG_NHWC, false>(x, b, bl, y, act_table, p, ab, s);
    return launch_act_scaled<WG_NCHW, false>(x, b, bl, y, act_table, p, ab, s);
}

}  // namespace wg
