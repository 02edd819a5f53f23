// Winograd-domain contraction M[e][t][k] = sum_c W[e][k][c] * D[e][t][c] at the 26
// free entries (Section 3.4): 16 real and 10 complex products per tile and
// channel pair, each complex one by the three-multiplication rule of Section
// 3.1, with the partial products kept apart until the channel sum is complete.
// Every real product of two 12-bit operands is three int8 matrix-core products
// (limb-level Karatsuba, Section 3.1), accumulated in int32 and recombined once.
// In scaled mode (Section 4.2) the filters are single int8 limbs and the
// reciprocal r/2^q is applied to the finished sums.
#include "subproducts.h"

namespace wg {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// grid: (tile blocks of 64, filter blocks of 64, 26 entries); 4 waves, each a 32x32 block
// computed with v_mfma_i32_32x32x32_i8: tiles are the rows, filters the columns, so a lane
// holds one filter column and its stores run along K.
template <int MODE>
__global__ __launch_bounds__(256) void contraction_kernel(const int8_t* __restrict__ V,
                                                          const uint8_t* __restrict__ blob,
                                                          size_t table_off, size_t planes_off,
                                                          int32_t* __restrict__ M, Problem p) {
    if (!blob_matches(reinterpret_cast<const BlobHeader*>(blob), p.K, p.C, MODE)) return;
    const int8_t* U = reinterpret_cast<const int8_t*>(blob + planes_off);
    const int entry = blockIdx.z;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int t0 = blockIdx.x * 64 + (wave & 1) * 32;
    const int k0 = blockIdx.y * 64 + (wave >> 1) * 32;
    const int row = lane & 31, half = lane >> 5;
    constexpr int NP = MODE == WG_LOSSLESS ? 138 : 46;
    const size_t a_cb = (size_t)p.Tp * kCBlock, b_cb = (size_t)(p.Kp >> 4) * NP * kFilterFragBytes;

    v16i re = {0}, im = {0};
    const int nsub = num_subproducts<MODE>(entry);
    for (int s = 0; s < nsub; ++s) {
        const SubProduct sp = subproduct<MODE>(entry, s);
        const int8_t* A = V + ((size_t)sp.a_plane * p.CB * p.Tp + t0 + row) * kCBlock + half * 16;
        const int8_t* B = U + filter_plane_offset(sp.b_plane, 0, k0 + row, half * 16, p.Kp, NP);
        v16i acc = {0};
        for (int cb = 0; cb < p.CB; ++cb) {
            v4i a0 = *reinterpret_cast<const v4i*>(A + cb * a_cb);
            v4i a1 = *reinterpret_cast<const v4i*>(A + cb * a_cb + 32);
            v4i b0 = *reinterpret_cast<const v4i*>(B + cb * b_cb);
            v4i b1 = *reinterpret_cast<const v4i*>(B + cb * b_cb + 32);
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, acc, 0, 0, 0);
        }
        // |acc| <= 94*94*896 < 2^23: the 24-bit multiply-add is exact modulo 2^32
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            re[i] += __mul24(acc[i], sp.w_re);
            im[i] += __mul24(acc[i], sp.w_im);
        }
    }

    const int k = k0 + row;
    if (MODE == WG_SCALED) {
        // reverse scaling (Section 4.2): (m * r + 2^(q-1)) >> q, 64-bit intermediate
        const ScaleEntry* table = reinterpret_cast<const ScaleEntry*>(blob + table_off);
        const ScaleEntry se = table[(size_t)k * kEntries + entry];
        if (se.n != 0) {
            const long long rnd = se.q > 0 ? (1ll << (se.q - 1)) : 0ll;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                re[i] = (int)(((long long)re[i] * se.r + rnd) >> se.q);
                im[i] = (int)(((long long)im[i] * se.r + rnd) >> se.q);
            }
        }
    }

    if (k >= p.K) return;
    const int plane_re = entry < kRealEntries ? entry : kRealEntries + 2 * (entry - kRealEntries);
    int32_t* Mre = M + (size_t)plane_re * p.Tp * p.Kp + k;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int t = t0 + 8 * (i / 4) + 4 * half + (i % 4);
        if (t < p.T) {
            Mre[(size_t)t * p.Kp] = re[i];
            if (entry >= kRealEntries) Mre[(size_t)p.Tp * p.Kp + (size_t)t * p.Kp] = im[i];
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

}  // namespace

hipError_t launch_contraction(const int8_t* V, const void* blob, int32_t* M, const Problem& p, int mode,
                              hipStream_t s) {
    const BlobLayout bl = blob_layout(p.Kp, p.CB, mode);
    dim3 grid(p.Tp / 64, p.Kp / 64, kEntries);
    const uint8_t* b = static_cast<const uint8_t*>(blob);
    if (mode == WG_LOSSLESS)
        contraction_kernel<WG_LOSSLESS><<<grid, 256, 0, s>>>(V, b, bl.table_off, bl.planes_off, M, p);
    else
        contraction_kernel<WG_SCALED><<<grid, 256, 0, s>>>(V, b, bl.table_off, bl.planes_off, M, p);
    return hipGetLastError();
}

hipError_t launch_unpack_accumulators(const int32_t* M, int32_t* dense, const Problem& p, hipStream_t s) {
    size_t total = (size_t)kAccPlanes * p.T * p.K;
    unpack_accumulators_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(M, dense, p);
    return hipGetLastError();
}

}  // namespace wg
