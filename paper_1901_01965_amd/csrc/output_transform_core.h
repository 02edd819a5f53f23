// The arithmetic of the output transform Y = A^T M A (Section 3.3) on the 26 free entries of
// the conjugate-symmetric accumulator tile (Section 3.4), for one thread that holds all of
// them; shared by the stand-alone output transform and the narrow-input kernel.
#pragma once
#include <hip/hip_runtime.h>

namespace wg {

// Row rule of A^T on (m0, m1, m2, m3, conj(m3), m5) with m0,m1,m2,m5 real:
//   y0 = m0+m1+m2+2Re m3, y1 = m1-m2-2Im m3, y2 = m1+m2-2Re m3, y3 = m1-m2+2Im m3+m5
__device__ inline void at_rule(int m0, int m1, int m2, int m3r, int m3i, int m5, int y[4]) {
    const int s = m1 + m2, d = m1 - m2;
    y[0] = m0 + s + 2 * m3r;
    y[1] = d - 2 * m3i;
    y[2] = s - 2 * m3r;
    y[3] = d + 2 * m3i + m5;
}

// re[4 ri + ci] = M[r][c] for r, c in {0,1,2,5}; complex cr/ci[0..3] = M[{0,1,2,5}][3],
// [4..7] = M[3][{0,1,2,5}], [8] = M[3][3], [9] = M[3][4].  out[j][i] = 16 Y[i][j] (the caller
// applies the rescale by 2^-4).
__device__ inline void output_tile(const int re[16], const int cr[10], const int ci[10], int out[4][4]) {
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
#pragma unroll
    for (int j = 0; j < 4; ++j) at_rule(z[0][j], z[1][j], z[2][j], z3r[j], z3i[j], z[3][j], out[j]);
}

}  // namespace wg
