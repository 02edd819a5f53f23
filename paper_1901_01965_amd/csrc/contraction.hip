// Winograd-domain contraction M[e][t][k] = sum_c W[e][k][c] * D[e][t][c] at the 26
// free entries (Section 3.4): 16 real and 10 complex products per tile and
// channel pair, each complex one by the three-multiplication rule of Section
// 3.1, with the partial products kept apart until the channel sum is complete.
// Every real product of two 12-bit operands is three int8 matrix-core products
// (limb-level Karatsuba, Section 3.1), accumulated in int32 and recombined once.
// In scaled mode (Section 4.2) the filters are single int8 limbs and the
// reciprocal r/2^q is applied to the finished sums.
//
// One workgroup owns one entry and a 128-tile x 128-filter block of it.  Each of
// the entry's sub-products is a [128 x C] x [C x 128] int8 GEMM.  Operand blocks
// of 64 channels travel from L2 straight into a four-stage LDS ring
// (global_load_lds_dwordx4, no register staging), three stages ahead of the
// matrix cores; every wave keeps a 64x64 block of v_mfma_i32_32x32x32_i8
// accumulators; the finished channel sum is folded into Re/Im with the
// sub-product's integer weights.
#include "subproducts.h"

namespace wg {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBlockTiles = 128, kBlockFilters = 128;
constexpr int kOperandBytes = 128 * kCBlock;        // one staged operand block: 128 rows x 64 bytes
constexpr int kStageBytes = 2 * kOperandBytes;      // activations + filters
constexpr int kStages = 4;
constexpr int kContractionLds = kStages * kStageBytes;   // 64 KB

// A staged row keeps its 64 bytes but stores 16-byte chunk c at position c ^ swizzle(row), which
// spreads the fragment reads of 16 consecutive rows over all banks.  The permutation is applied
// on the global side: the LDS side of a direct load is fixed (lane l lands at base + 16 l).
__device__ inline int swizzle(int row) { return (row ^ (row >> 2)) & 3; }

template <int MODE>
struct BlockLoader {
    const int8_t* V;
    const int8_t* U;
    size_t a_plane_stride, a_cb_stride, b_cb_stride;
    int a_off[2], b_off[2];   // this lane's source offsets inside plane 0, channel block 0
    int lds_off[2];           // wave-uniform destination of each instruction inside an operand block

    // wave w fills rows 32w..32w+31 of both operand blocks: two instructions of 16 rows each
    __device__ inline void init(const int8_t* V_, const int8_t* U_, const Problem& p, int t0, int k0, int wave,
                                int lane) {
        constexpr int NP = MODE == WG_LOSSLESS ? 138 : 46;
        V = V_; U = U_;
        a_plane_stride = (size_t)p.CB * p.Tp * kCBlock;
        a_cb_stride = (size_t)p.Tp * kCBlock;
        b_cb_stride = (size_t)(p.Kp >> 4) * NP * kFilterFragBytes;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = wave * 32 + i * 16 + (lane >> 2);
            const int chunk = (lane & 3) ^ swizzle(row);
            // rows beyond the padded extent are clamped: their products are never stored
            const int t = min(t0 + row, p.Tp - 1), k = min(k0 + row, p.Kp - 1);
            a_off[i] = t * kCBlock + chunk * 16;
            b_off[i] = (int)filter_plane_offset(0, 0, k, chunk * 16, p.Kp, NP);
            lds_off[i] = (wave * 32 + i * 16) * kCBlock;
        }
    }
    __device__ inline void issue(int8_t* stage, int a_plane, int b_plane, int cb) const {
        const int8_t* A = V + a_plane * a_plane_stride + cb * a_cb_stride;
        const int8_t* B = U + cb * b_cb_stride + (size_t)b_plane * kFilterFragBytes;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            __builtin_amdgcn_global_load_lds(A + a_off[i], stage + lds_off[i], 16, 0, 0);
            __builtin_amdgcn_global_load_lds(B + b_off[i], stage + kOperandBytes + lds_off[i], 16, 0, 0);
        }
    }
};

// 64 channels of one staged block into the wave's 2x2 accumulators.  a_row/b_row: byte offset of
// this lane's row (lane % 32) in each operand block; sw = swizzle of that row (the same for the
// row 32 further on); half = lane / 32 selects the 16-byte half of a 32-channel step.
template <bool FIRST>
__device__ inline void mma_block(const int8_t* stage, int a_row, int b_row, int sw_a, int sw_b, int half,
                                 v16i (&acc)[2][2]) {
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        v4i a[2], b[2];
        const int ca = ((2 * ks + half) ^ sw_a) * 16, cbb = ((2 * ks + half) ^ sw_b) * 16;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            a[i] = *reinterpret_cast<const v4i*>(stage + a_row + i * 32 * kCBlock + ca);
            b[i] = *reinterpret_cast<const v4i*>(stage + kOperandBytes + b_row + i * 32 * kCBlock + cbb);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if (FIRST && ks == 0) {
                    constexpr v16i zero = {0};
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], zero, 0, 0, 0);
                } else {
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
                }
            }
    }
}

// grid: (ceil(T/128), ceil(K/128), 26 entries), complex entries (nine sub-products) first.
template <int MODE>
__global__ __launch_bounds__(256) void contraction_kernel(const int8_t* __restrict__ V,
                                                          const uint8_t* __restrict__ blob,
                                                          size_t table_off, size_t planes_off,
                                                          int32_t* __restrict__ M, Problem p) {
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    if (!blob_matches(reinterpret_cast<const BlobHeader*>(blob), p.K, p.C, MODE)) return;
    const int entry = kEntries - 1 - (int)blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int t0 = blockIdx.x * kBlockTiles, k0 = blockIdx.y * kBlockFilters;
    const int wm = wave & 1, wn = wave >> 1;

    BlockLoader<MODE> loader;
    loader.init(V, reinterpret_cast<const int8_t*>(blob + planes_off), p, t0, k0, wave, lane);
    const int a_row = (wm * 64 + (lane & 31)) * kCBlock, b_row = (wn * 64 + (lane & 31)) * kCBlock;
    const int sw_a = swizzle(wm * 64 + (lane & 31)), sw_b = swizzle(wn * 64 + (lane & 31)), half = lane >> 5;

    v16i re[2][2], im[2][2], acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) { re[i][j] = (v16i){0}; im[i][j] = (v16i){0}; }

    const int nsub = entry < kRealEntries ? num_subproducts<MODE>(0) : num_subproducts<MODE>(kRealEntries);
    const int total = nsub * p.CB;
    // stage f of the stream = (sub-product f / CB, channel block f % CB); fill the first three
    int fs = 0, fcb = 0;   // sub-product and channel block of the next stage to request
    auto request = [&](int f) {
        const SubProduct sp = subproduct<MODE>(entry, fs);
        loader.issue(lds + (f % kStages) * kStageBytes, sp.a_plane, sp.b_plane, fcb);
        if (++fcb == p.CB) { fcb = 0; ++fs; }
    };
    for (int f = 0; f < kStages - 1; ++f) {
        if (f < total) request(f);
    }
    int it = 0;
    for (int s = 0; s < nsub; ++s) {
        const SubProduct sp = subproduct<MODE>(entry, s);
        for (int cb = 0; cb < p.CB; ++cb, ++it) {
            // stage `it` has landed once at most the requests of the stages after it are pending
            const int later = min(total - 1 - it, kStages - 2);
            if (later >= 2)      asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
            else if (later == 1) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            else                 asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();   // all parts of stage `it` are in LDS; stage it-1 is no longer read
            if (it + kStages - 1 < total) request(it + kStages - 1);
            const int8_t* stage = lds + (it % kStages) * kStageBytes;
            if (cb == 0) mma_block<true>(stage, a_row, b_row, sw_a, sw_b, half, acc);
            else         mma_block<false>(stage, a_row, b_row, sw_a, sw_b, half, acc);
        }
        // |acc| <= 94*94*896 < 2^23: the 24-bit multiply-add is exact modulo 2^32
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    re[i][j][r] += __mul24(acc[i][j][r], sp.w_re);
                    im[i][j][r] += __mul24(acc[i][j][r], sp.w_im);
                }
    }

    const int plane_re = entry < kRealEntries ? entry : kRealEntries + 2 * (entry - kRealEntries);
    const size_t plane = (size_t)p.Tp * p.Kp;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int k = k0 + wn * 64 + j * 32 + (lane & 31);
        ScaleEntry se = {0, 0, 1, 0};
        if (MODE == WG_SCALED && k < p.Kp)
            se = reinterpret_cast<const ScaleEntry*>(blob + table_off)[(size_t)k * kEntries + entry];
        const long long rnd = se.q > 0 ? (1ll << (se.q - 1)) : 0ll;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int vr = re[i][j][r], vi = im[i][j][r];
                if (MODE == WG_SCALED && se.n != 0) {
                    // reverse scaling (Section 4.2): (m * r + 2^(q-1)) >> q, 64-bit intermediate
                    vr = (int)(((long long)vr * se.r + rnd) >> se.q);
                    vi = (int)(((long long)vi * se.r + rnd) >> se.q);
                }
                const int t = t0 + wm * 64 + i * 32 + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
                if (t < p.T && k < p.K) {
                    int32_t* m = M + plane_re * plane + (size_t)t * p.Kp + k;
                    m[0] = vr;
                    if (entry >= kRealEntries) m[plane] = vi;
                }
            }
        }
    }
}

__global__ void unpack_accumulators_kernel(const int32_t* M, int32_t* dense, Problem p) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)kAccPlanes * p.T * p.K;
    if (i >= total) return;
    int k = (int)(i % p.K);
    int t = (int)((i / p.K) % p.T);
    int pl = (int)(i / ((size_t)p.K * p.T));
    dense[i] = M[((size_t)pl * p.Tp + t) * p.Kp + k];
}

template <int MODE>
hipError_t configure_contraction() {
    static bool done = false;
    if (done) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&contraction_kernel<MODE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kContractionLds);
    done = e == hipSuccess;
    return e;
}

}  // namespace

hipError_t launch_contraction(const int8_t* V, const void* blob, int32_t* M, const Problem& p, int mode,
                              hipStream_t s) {
    if (hipError_t e = mode == WG_LOSSLESS ? configure_contraction<WG_LOSSLESS>() : configure_contraction<WG_SCALED>())
        return e;
    const BlobLayout bl = blob_layout(p.Kp, p.CB, mode);
    dim3 grid(ceil_div(p.T, kBlockTiles), ceil_div(p.K, kBlockFilters), kEntries);
    const uint8_t* b = static_cast<const uint8_t*>(blob);
    if (mode == WG_LOSSLESS)
        contraction_kernel<WG_LOSSLESS><<<grid, 256, kContractionLds, s>>>(V, b, bl.table_off, bl.planes_off, M, p);
    else
        contraction_kernel<WG_SCALED><<<grid, 256, kContractionLds, s>>>(V, b, bl.table_off, bl.planes_off, M, p);
    return hipGetLastError();
}

hipError_t launch_unpack_accumulators(const int32_t* M, int32_t* dense, const Problem& p, hipStream_t s) {
    size_t total = (size_t)kAccPlanes * p.T * p.K;
    unpack_accumulators_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(M, dense, p);
    return hipGetLastError();
}

}  // namespace wg
