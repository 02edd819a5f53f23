// Output transform Y = A^T M A (Section 3.3) on the conjugate-symmetric
// accumulator tile (Section 3.4): only real parts are formed, since the
// imaginary parts of the result vanish; then the rescale by 2^-4 that undoes
// G' = 4G on both sides (the analogue of the shift after each final transform
// that Section 4.2 describes for G' = 2G).
#include "wg_internal.h"

namespace wg {
namespace {

// Row rule of A^T on (m0, m1, m2, m3, conj(m3), m5) with m0,m1,m2,m5 real:
//   y0 = m0+m1+m2+2Re m3, y1 = m1-m2-2Im m3, y2 = m1+m2-2Re m3, y3 = m1-m2+2Im m3+m5
__device__ inline void at_rule(int m0, int m1, int m2, int m3r, int m3i, int m5, int y[4]) {
    const int s = m1 + m2, d = m1 - m2;
    y[0] = m0 + s + 2 * m3r;
    y[1] = d - 2 * m3i;
    y[2] = s - 2 * m3r;
    y[3] = d + 2 * m3i + m5;
}

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

    // Z = M A: rows 0,1,2,5 are real; row 3 is complex (row 4 is its conjugate)
    int z[4][4];
#pragma unroll
    for (int ri = 0; ri < 4; ++ri)
        at_rule(re[4 * ri], re[4 * ri + 1], re[4 * ri + 2], cr[ri], ci[ri], re[4 * ri + 3], z[ri]);
    // row 3: e_c = M[3][c] for c in {0,1,2,5} (cr/ci[4..7]), e3 = M[3][3], e4 = M[3][4]
    int z3r[4], z3i[4];
    {
        const int sr = cr[8] + cr[9], si = ci[8] + ci[9];   // e3 + e4
        const int dr = cr[8] - cr[9], di = ci[8] - ci[9];   // e3 - e4
        const int ar = cr[5] + cr[6], ai = ci[5] + ci[6];   // e1 + e2
        const int br = cr[5] - cr[6], bi = ci[5] - ci[6];   // e1 - e2
        z3r[0] = cr[4] + ar + sr;        z3i[0] = ci[4] + ai + si;
        z3r[1] = br - di;                z3i[1] = bi + dr;          // (e1-e2) + i (e3-e4)
        z3r[2] = ar - sr;                z3i[2] = ai - si;
        z3r[3] = br + di + cr[7];        z3i[3] = bi - dr + ci[7];  // (e1-e2) - i (e3-e4) + e5
    }

    int n, ty, tx;
    decode_tile(p, t, n, ty, tx);
    const int rnd = MODE == WG_SCALED ? 8 : 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int col[4];
        at_rule(z[0][j], z[1][j], z[2][j], z3r[j], z3i[j], z[3][j], col);
        const int w = 4 * tx + j;
        if (w >= p.W) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int h = 4 * ty + i;
            if (h >= p.H) continue;
            const int v = (col[i] + rnd) >> 4;
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
