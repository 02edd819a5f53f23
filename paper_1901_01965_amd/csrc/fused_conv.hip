// The whole hot path in one kernel: input transform (Section 3.3-3.4) of a block
// of 16 tiles into int8 operand planes held in LDS, the Winograd-domain
// products of Section 3.4 against 32 filters on the int8 matrix cores, and the
// output transform accumulated on the fly, so neither the transformed
// activations nor the 36 accumulator planes ever travel through HBM.
//
// The output transform Y = A^T M A is linear in M, and M is a sum over input
// channels, so each finished row of M (for one 64-channel block) is reduced by
// the row rule of A^T at once and added into the 16 outputs of the tile.  That is
// valid for any number of channel blocks in lossless mode; the reverse scaling of
// Section 4.2 is not linear (it rounds), so scaled mode uses this kernel only
// when all input channels fit one block.
#include "input_transform_core.h"
#include <type_traits>
#include <utility>

#include "subproducts.h"

namespace wg {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kFusedTiles = 16;     // tiles per workgroup (rows of the 16x16x64 matrix-core product)
constexpr int kFusedFilters = 32;   // filters per workgroup: two 16-wide column blocks
constexpr int kPlaneBytes = kFusedTiles * kCBlock;   // one operand plane of the tile block in LDS

// LDS operand plane: the 16-byte piece holding 16 consecutive channels (group c16) of a tile
// sits in slot c16*16 + ((tile + 4*c16) & 15); lane l of a wave reads slot(l/16, l%16), which
// tiles the plane without bank conflicts for the 4-byte writes as well as the 16-byte reads.
__device__ inline int lds_slot(int c16, int tile) { return c16 * 16 + ((tile + 4 * c16) & 15); }

struct LdsPlaneSink {
    int8_t* base;
    __device__ inline void put(int plane, s8x4 bytes) const {
        *reinterpret_cast<s8x4*>(base + plane * kPlaneBytes) = bytes;
    }
};

struct LaneContext {
    const int8_t* a_lds;        // this lane's 16-byte slot in plane 0
    const int8_t* b_glob;       // this lane's 16 bytes of filter plane 0, current channel block
    size_t b_plane_stride;      // bytes between filter planes
    const ScaleEntry* table_k;  // scaling table row of this lane's filter (scaled mode)
};

// compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(<N-1>)
template <class F, int... Is>
__device__ inline void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ inline void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// The sub-products one wave issues, in order.  Half 0 owns rows 0,1,2 of M, half 1 rows 5
// and 3.  A real row RI (rows 0,1,2,5) holds entries 4RI..4RI+3 and the complex entry 16+RI;
// the complex row holds entries 20..25.
struct Step {
    int entry, sub;      // which entry, which of its sub-products
    int row;             // 0..3: real row RI, 4: the complex row
    int pos;             // position of the entry within its row
    bool last_sub;       // last sub-product of the entry
    bool last_in_row;    // ... and last entry of the row
};
__host__ __device__ constexpr int row_entries(int row) { return row < 4 ? 5 : 6; }
__host__ __device__ constexpr int row_entry(int row, int pos) {
    return row < 4 ? (pos < 4 ? 4 * row + pos : kRealEntries + row) : kRealEntries + 4 + pos;
}
__host__ __device__ constexpr int half_rows(int half) { return half == 0 ? 3 : 2; }
__host__ __device__ constexpr int half_row(int half, int i) { return half == 0 ? i : (i == 0 ? 3 : 4); }

template <int MODE, int HALF>
__host__ __device__ constexpr int sequence_length() {
    int n = 0;
    for (int r = 0; r < half_rows(HALF); ++r)
        for (int e = 0; e < row_entries(half_row(HALF, r)); ++e)
            n += num_subproducts<MODE>(row_entry(half_row(HALF, r), e));
    return n;
}
template <int MODE, int HALF>
__host__ __device__ constexpr Step sequence_step(int i) {
    int n = 0;
    for (int r = 0; r < half_rows(HALF); ++r) {
        const int row = half_row(HALF, r);
        for (int e = 0; e < row_entries(row); ++e) {
            const int entry = row_entry(row, e), ns = num_subproducts<MODE>(entry);
            if (i < n + ns) {
                const bool last = (i - n) == ns - 1;
                return Step{entry, i - n, row, e, last, last && e == row_entries(row) - 1};
            }
            n += ns;
        }
    }
    return Step{0, 0, 0, 0, false, false};
}

// Row rule of A^T on (m0, m1, m2, m3, conj(m3), m5) with m0,m1,m2,m5 real:
//   z0 = m0+m1+m2+2Re m3, z1 = m1-m2-2Im m3, z2 = m1+m2-2Re m3, z3 = m1-m2+2Im m3+m5
__device__ inline void at_rule(v4i m0, v4i m1, v4i m2, v4i m3r, v4i m3i, v4i m5, v4i z[4]) {
    const v4i s = m1 + m2, d = m1 - m2;
    z[0] = m0 + s + 2 * m3r;
    z[1] = d - 2 * m3i;
    z[2] = s - 2 * m3r;
    z[3] = d + 2 * m3i + m5;
}

// A finished row of M is reduced by the row rule and enters the 16 outputs with the
// column-rule coefficients of A^T.  Real rows 0,1,2,5 (ROW = 0..3; entries m0,m1,m2,m5 real
// at positions 0..3, complex m3 at position 4): row 0 -> y0; rows 1, 2 -> (+,+,+,+), (+,-,+,-);
// row 5 -> y3.  The complex row 3 (ROW = 4; e0,e1,e2,e5 at positions 0..3, e3 = M[3][3] and
// e4 = M[3][4] at 4, 5; row 4 of M is its conjugate): y0 += 2Re z, y1 -= 2Im z, y2 -= 2Re z,
// y3 += 2Im z.
template <int ROW>
__device__ inline void finish_row(const v4i (&er)[6], const v4i (&ei)[6], v4i (&Y)[16]) {
    if constexpr (ROW < 4) {
        v4i z[4];
        at_rule(er[0], er[1], er[2], er[4], ei[4], er[3], z);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (ROW == 0) Y[j] += z[j];
            if (ROW == 1) { Y[j] += z[j]; Y[4 + j] += z[j]; Y[8 + j] += z[j]; Y[12 + j] += z[j]; }
            if (ROW == 2) { Y[j] += z[j]; Y[4 + j] -= z[j]; Y[8 + j] += z[j]; Y[12 + j] -= z[j]; }
            if (ROW == 3) Y[12 + j] += z[j];
        }
    } else {
        const v4i sr = er[4] + er[5], si = ei[4] + ei[5], dr = er[4] - er[5], di = ei[4] - ei[5];
        const v4i ar = er[1] + er[2], ai = ei[1] + ei[2], br = er[1] - er[2], bi = ei[1] - ei[2];
        v4i zr[4], zi[4];
        zr[0] = er[0] + ar + sr;   zi[0] = ei[0] + ai + si;
        zr[1] = br - di;           zi[1] = bi + dr;            // (e1-e2) + i (e3-e4)
        zr[2] = ar - sr;           zi[2] = ai - si;
        zr[3] = br + di + er[3];   zi[3] = bi - dr + ei[3];    // (e1-e2) - i (e3-e4) + e5
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            Y[j] += 2 * zr[j];
            Y[4 + j] -= 2 * zi[j];
            Y[8 + j] -= 2 * zr[j];
            Y[12 + j] += 2 * zi[j];
        }
    }
}

constexpr int kFilterPrefetch = 16;   // filter fragments in flight per wave (L2 latency cover)
constexpr int kLdsPrefetch = 2;       // activation fragments in flight from LDS

template <int MODE, int HALF>
struct ProductPhase {
    static constexpr int N = sequence_length<MODE, HALF>();
    v4i bring[kFilterPrefetch];

    __device__ inline static v4i load_b(const LaneContext& cx, int i) {
        const Step st = sequence_step<MODE, HALF>(i);
        const SubProduct sp = subproduct<MODE>(st.entry, st.sub);
        return *reinterpret_cast<const v4i*>(cx.b_glob + (size_t)sp.b_plane * cx.b_plane_stride);
    }
    __device__ inline static v4i load_a(const LaneContext& cx, int i) {
        const Step st = sequence_step<MODE, HALF>(i);
        const SubProduct sp = subproduct<MODE>(st.entry, st.sub);
        return *reinterpret_cast<const v4i*>(cx.a_lds + sp.a_plane * kPlaneBytes);
    }

    // Filter fragments do not depend on the transform phase: start them before it.
    __device__ inline void prefetch(const LaneContext& cx) {
        static_for<kFilterPrefetch>([&](auto I) {
            if constexpr (I < N) bring[I] = load_b(cx, I);
        });
    }

    // One 64-channel block of this wave's rows: every sub-product is a single 16x16x64
    // matrix-core instruction (channel sum complete within the block); its result is weighted
    // into Re/Im of its entry one step later, while the next instruction runs.
    __device__ inline void run(const LaneContext& cx, v4i (&Y)[16]) {
        v4i aring[kLdsPrefetch];
        static_for<kLdsPrefetch>([&](auto I) { aring[I] = load_a(cx, I); });
        v4i re = {0, 0, 0, 0}, im = {0, 0, 0, 0}, acc_prev = {0, 0, 0, 0};
        v4i er[6], ei[6];
        static_for<N + 1>([&](auto I) {
            constexpr int i = I;
            v4i acc_cur = {0, 0, 0, 0};
            if constexpr (i < N) {
                const v4i a = aring[i % kLdsPrefetch], b = bring[i % kFilterPrefetch];
                constexpr v4i zero = {0, 0, 0, 0};
                acc_cur = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, zero, 0, 0, 0);
                if constexpr (i + kLdsPrefetch < N) aring[i % kLdsPrefetch] = load_a(cx, i + kLdsPrefetch);
                if constexpr (i + kFilterPrefetch < N) bring[i % kFilterPrefetch] = load_b(cx, i + kFilterPrefetch);
            }
            if constexpr (i > 0) {
                constexpr Step st = sequence_step<MODE, HALF>(i - 1);
                constexpr SubProduct sp = subproduct<MODE>(st.entry, st.sub);
                if constexpr (st.sub == 0) { re = (v4i){0, 0, 0, 0}; im = (v4i){0, 0, 0, 0}; }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (sp.w_re != 0) re[q] += __mul24(acc_prev[q], sp.w_re);
                    if (sp.w_im != 0) im[q] += __mul24(acc_prev[q], sp.w_im);
                }
                if constexpr (st.last_sub) {
                    if constexpr (MODE == WG_SCALED) {
                        // reverse scaling (Section 4.2): (m * r + 2^(q-1)) >> q, 64-bit intermediate
                        const ScaleEntry se = cx.table_k[st.entry];
                        if (se.n != 0) {
                            const long long rnd = se.q > 0 ? (1ll << (se.q - 1)) : 0ll;
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                re[q] = (int)(((long long)re[q] * se.r + rnd) >> se.q);
                                im[q] = (int)(((long long)im[q] * se.r + rnd) >> se.q);
                            }
                        }
                    }
                    er[st.pos] = re;
                    ei[st.pos] = im;
                    if constexpr (st.last_in_row) finish_row<st.row>(er, ei, Y);
                }
            }
            acc_prev = acc_cur;
            __builtin_amdgcn_sched_barrier(0);
        });
    }
};

// grid: (ceil(T/16), Kp/32).  256 threads: in the transform phase one thread per (tile,
// four channels); in the product phase wave w owns filter block (w & 1) and half of the
// rows of M (w >> 1: rows 0,1,2 or rows 5,3); the two halves are added through LDS.
template <int LAYOUT, bool VEC4, int MODE>
__global__ __launch_bounds__(256) void fused_conv_kernel(const int8_t* __restrict__ x,
                                                         const uint8_t* __restrict__ blob, size_t table_off,
                                                         size_t planes_off, int32_t* __restrict__ y, Problem p) {
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    if (!blob_matches(reinterpret_cast<const BlobHeader*>(blob), p.K, p.C, MODE)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kblock = wave & 1, half = wave >> 1;
    const int tile0 = blockIdx.x * kFusedTiles;
    const int k = blockIdx.y * kFusedFilters + kblock * 16 + (lane & 15);

    // transform-phase identity
    const int a_tile = tid >> 4, a_cq = tid & 15;
    const int a_t = tile0 + a_tile;
    const int a_tx = a_t % p.TW, a_ty = (a_t / p.TW) % p.TH, a_n = a_t / (p.TW * p.TH);
    OperandSplitter<MODE, LdsPlaneSink> out;
    out.sink.base = lds + lds_slot(a_cq >> 2, a_tile) * 16 + (a_cq & 3) * 4;

    LaneContext cx;
    cx.a_lds = lds + lds_slot(lane >> 4, lane & 15) * 16;
    cx.b_plane_stride = (size_t)p.CB * p.Kp * kCBlock;
    cx.table_k = reinterpret_cast<const ScaleEntry*>(blob + table_off) + (size_t)k * kEntries;
    const int8_t* b_lane = reinterpret_cast<const int8_t*>(blob + planes_off) + (size_t)k * kCBlock + (lane >> 4) * 16;

    v4i Y[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) Y[i] = (v4i){0, 0, 0, 0};

    ProductPhase<MODE, 0> phase0;
    ProductPhase<MODE, 1> phase1;
    for (int cb = 0; cb < p.CB; ++cb) {
        cx.b_glob = b_lane + (size_t)cb * p.Kp * kCBlock;
        if (half == 0) phase0.prefetch(cx); else phase1.prefetch(cx);
        if (cb > 0) __syncthreads();   // everyone is done reading the previous block's planes
        if (a_t < p.T) transform_tile<LAYOUT, VEC4, MODE>(x, p, a_n, a_ty, a_tx, cb * kCBlock + 4 * a_cq, out);
        __syncthreads();
        if (half == 0) phase0.run(cx, Y); else phase1.run(cx, Y);
    }

    // add the two halves: waves 2,3 park their partial outputs in LDS, waves 0,1 finish
    __syncthreads();
    v4i* park = reinterpret_cast<v4i*>(lds) + (kblock * 16) * 64 + lane;
    if (half == 1) {
#pragma unroll
        for (int i = 0; i < 16; ++i) park[i * 64] = Y[i];
    }
    __syncthreads();
    if (half == 1 || k >= p.K) return;
#pragma unroll
    for (int i = 0; i < 16; ++i) Y[i] += park[i * 64];

    const int rnd = MODE == WG_SCALED ? 8 : 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int t = tile0 + 4 * (lane >> 4) + q;     // row of the matrix-core result held in register q
        if (t >= p.T) continue;
        const int tx = t % p.TW, ty = (t / p.TW) % p.TH, n = t / (p.TW * p.TH);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int h = 4 * ty + i;
            if (h >= p.H) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int w = 4 * tx + j;
                if (w >= p.W) continue;
                const int v = (Y[4 * i + j][q] + rnd) >> 4;
                if (LAYOUT == WG_NHWC) y[(((size_t)n * p.H + h) * p.W + w) * p.K + k] = v;
                else                   y[(((size_t)n * p.K + k) * p.H + h) * p.W + w] = v;
            }
        }
    }
}

template <int LAYOUT, bool VEC4, int MODE>
hipError_t launch(const int8_t* x, const uint8_t* blob, const BlobLayout& bl, int32_t* y, const Problem& p,
                  hipStream_t s) {
    const size_t lds_bytes = (size_t)num_activation_planes(MODE) * kPlaneBytes;
    static bool configured = false;   // per template instance
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fused_conv_kernel<LAYOUT, VEC4, MODE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        configured = true;
    }
    dim3 grid(ceil_div(p.T, kFusedTiles), p.Kp / kFusedFilters);
    fused_conv_kernel<LAYOUT, VEC4, MODE><<<grid, 256, lds_bytes, s>>>(x, blob, bl.table_off, bl.planes_off, y, p);
    return hipGetLastError();
}

}  // namespace

bool fused_conv_supported(const Problem& p, int mode) { return mode == WG_LOSSLESS || p.CB == 1; }

hipError_t launch_fused_conv(const int8_t* x, const void* blob, int32_t* y, const Problem& p, int layout, int mode,
                             hipStream_t s) {
    const BlobLayout bl = blob_layout(p.Kp, p.CB, mode);
    const uint8_t* b = static_cast<const uint8_t*>(blob);
    if (layout == WG_NHWC && p.C % 4 == 0)
        return mode == WG_LOSSLESS ? launch<WG_NHWC, true, WG_LOSSLESS>(x, b, bl, y, p, s)
                                   : launch<WG_NHWC, true, WG_SCALED>(x, b, bl, y, p, s);
    if (layout == WG_NHWC)
        return mode == WG_LOSSLESS ? launch<WG_NHWC, false, WG_LOSSLESS>(x, b, bl, y, p, s)
                                   : launch<WG_NHWC, false, WG_SCALED>(x, b, bl, y, p, s);
    return mode == WG_LOSSLESS ? launch<WG_NCHW, false, WG_LOSSLESS>(x, b, bl, y, p, s)
                               : launch<WG_NCHW, false, WG_SCALED>(x, b, bl, y, p, s);
}

}  // namespace wg
