// Output transform Y = A^T M A (Section 3.3) on the conjugate-symmetric
// accumulator tile (Section 3.4): only real parts are formed, since the
// imaginary parts of the result vanish; then the rescale by 2^-4 that undoes
// G' = 4G on both sides (the analogue of the shift after each final transform
// that Section 4.2 describes for G' = 2G).
#include "output_transform_core.h"
#include "wg_internal.h"

namespace wg {
namespace {

// One thread per (tile, filter); lanes run along K so the 36 plane reads coalesce.
template <int LAYOUT, int MODE>
__global__ __launch_bounds__(256) void output_transform_kernel(const int32_t* __restrict__ M,
                                                               const uint8_t* __restrict__ blob,
                                                               int32_t* __restrict__ y, Problem p) {
    if (!blob_matches(reinterpret_cast<const BlobHeader*>(blob), p.K, p.C, MODE)) return;
    const int k = blockIdx.y * 64 + (threadIdx.x & 63);
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (k >= p.K || t >= p.T) return;
    const size_t plane = (size_t)p.Tp * p.Kp;
    const int32_t* m = M + (size_t)t * p.Kp + k;

    int re[16], cr[10], ci[10];
#pragma unroll
    for (int e = 0; e < 16; ++e) re[e] = m[e * plane];
#pragma unroll
    for (int j = 0; j < 10; ++j) {
        if (MODE == WG_LOSSLESS) {
            // the contraction keeps the three real products of a complex entry apart (Section 3.4);
            // Re = P1 - P2, Im = P3 - P1 - P2 (Section 3.1), formed here after the channel sum
            const int p1 = m[(16 + 3 * j) * plane], p2 = m[(17 + 3 * j) * plane], p3 = m[(18 + 3 * j) * plane];
            cr[j] = p1 - p2;
            ci[j] = p3 - p1 - p2;
        } else {
            cr[j] = m[(16 + 2 * j) * plane];
            ci[j] = m[(17 + 2 * j) * plane];
        }
    }

    int out[4][4];   // out[j][i]: output row i, column j
    output_tile(re, cr, ci, out);

    int n, ty, tx;
    decode_tile(p, t, n, ty, tx);
    const int rnd = MODE == WG_SCALED ? 8 : 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int w = 4 * tx + j;
        if (w >= p.W) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int h = 4 * ty + i;
            if (h >= p.H) continue;
            const int v = (out[j][i] + rnd) >> 4;
            if (LAYOUT == WG_NHWC) y[(((size_t)n * p.H + h) * p.W + w) * p.K + k] = v;
            else                   y[(((size_t)n * p.K + k) * p.H + h) * p.W + w] = v;
        }
    }
}

}  // namespace

hipError_t launch_output_transform(const int32_t* M, const void* blob, int32_t* y, const Problem& p,
                                   int layout, int mode, hipStream_t s) {
    dim3 grid(ceil_div(p.T, 4), ceil_div(p.K, 64));
    const uint8_t* b = static_cast<const uint8_t*>(blob);
    if (layout == WG_NHWC) {
        if (mode == WG_LOSSLESS) output_transform_kernel<WG_NHWC, WG_LOSSLESS><<<grid, 256, 0, s>>>(M, b, y, p);
        else                     output_transform_kernel<WG_NHWC, WG_SCALED><<<grid, 256, 0, s>>>(M, b, y, p);
    } else {
        if (mode == WG_LOSSLESS) output_transform_kernel<WG_NCHW, WG_LOSSLESS><<<grid, 256, 0, s>>>(M, b, y, p);
        else                     output_transform_kernel<WG_NCHW, WG_SCALED><<<grid, 256, 0, s>>>(M, b, y, p);
    }
    return hipGetLastError();
}

}  // namespace wg
