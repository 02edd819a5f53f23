/*
 * CPU ORACLE -- test infrastructure, not product code.
 *
 * The rational Winograd algorithm F(2x2,3x3) in integer arithmetic, the running
 * example of Sections 4.1-4.2 of Meng & Brothers, "Efficient Winograd
 * Convolution via Integer Arithmetic" (SysML 2019) and the variant the paper's
 * own evaluation used (Section 4.4): filter transform with G' = 2G (the matrix
 * printed in Section 4.1), input transform B^T d B and output transform A^T m A
 * with the matrices of the minimal algorithm F(2,3) nested in two dimensions,
 * the filter precision scaling of Section 4.2 per output channel and X-Y
 * location, and the final rescale by 2^-2 that undoes G' = 2G on both sides.
 * Plain loops over the matrix definitions, int64 throughout.  Shares nothing
 * with the HIP library.
 *
 * Parity status (the pins live in tests/test_oracle_f2x2.py):
 *   oracle_f2_filter_transform  pinned: the printed G' and the printed expansion of
 *                               G' g G'^T in p_0..p_11 (Section 4.1); the printed
 *                               worst-case magnitude and bit-width tables
 *   oracle_f2_input_transform, oracle_f2_conv2d (lossless)
 *                               pinned: exact equality with the direct convolution,
 *                               1-D F(2,3) against brute force
 *   *_i16 variants              the same code on 16-bit inputs (uint8 minus zero point = int9,
 *                               Section 4.1); oracle_direct_conv2d_i16 pinned against the int8
 *                               direct convolution and a numpy einsum
 *   oracle_f2_conv2d (scaled)   special cases pinned (no location needs scaling
 *                               => equals lossless; scaled weights within the range;
 *                               table entries from the pinned factor routines);
 *                               the general lossy result is PARITY UNPINNED (the
 *                               paper prints no worked example of it).
 *   oracle_f2_scale_activations, oracle_f2_conv2d mode 2 (activations scaled as well)
 *                               Section 4.1 only remarks that the analysis of Section 4.2
 *                               carries over to B^T d B; the rule here is that section's
 *                               with the roles of filter and tile exchanged (see the
 *                               function).  Special cases pinned (no tile needs scaling
 *                               => equals mode 1; scaled activations within the range;
 *                               table entries from the pinned factor routines; the
 *                               operand a tile sees does not depend on the other tiles);
 *                               the general lossy result is PARITY UNPINNED.
 *
 * Tile t = (n*TH + ty)*TW + tx with TH = ceil(H/2), TW = ceil(W/2); tile (ty,tx)
 * reads input rows 2ty-1 .. 2ty+2, columns 2tx-1 .. 2tx+2 (zero outside: pad 1)
 * and owns outputs rows 2ty, 2ty+1, columns 2tx, 2tx+1.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* scaling routines of the main oracle file (same shared object) */
void oracle_scale_factor(int64_t mx, int64_t range, int32_t* n_out, int32_t* p_out);
void oracle_inverse_factor(int32_t n, int32_t p, int32_t* r_out, int32_t* q_out);
int64_t oracle_scale_round(int64_t v, int64_t mul, int sh);

/* F(2,3): y = A^T [ (G g) (.) (B^T d) ];  G' = 2G is the matrix printed in Section 4.1 */
static const int B2T[4][4] = {{1, 0, -1, 0}, {0, 1, 1, 0}, {0, -1, 1, 0}, {0, 1, 0, -1}};
static const int G2[4][3] = {{2, 0, 0}, {1, 1, 1}, {1, -1, 1}, {0, 0, 2}};
static const int A2T[2][4] = {{1, 1, 1, 0}, {0, 1, -1, -1}};

void oracle_f2_get_matrices(int8_t* bt /*[4][4]*/, int8_t* g2 /*[4][3]*/, int8_t* at /*[2][4]*/) {
    for (int r = 0; r < 4; ++r) for (int c = 0; c < 4; ++c) bt[r * 4 + c] = (int8_t)B2T[r][c];
    for (int r = 0; r < 4; ++r) for (int c = 0; c < 3; ++c) g2[r * 3 + c] = (int8_t)G2[r][c];
    for (int r = 0; r < 2; ++r) for (int c = 0; c < 4; ++c) at[r * 4 + c] = (int8_t)A2T[r][c];
}

static int cdiv(int a, int b) { return (a + b - 1) / b; }

/* The arithmetic below takes 16-bit inputs, so that it also covers the paper's own setting
   (Section 4.1): uint8 quantised values minus their zero point, i.e. int9 in [-255, 255].  The
   int8 entry points widen their arguments and call the same code. */
static int16_t* widen(const int8_t* a, size_t n) {
    int16_t* w = (int16_t*)malloc((n ? n : 1) * sizeof(int16_t));
    if (w) for (size_t i = 0; i < n; ++i) w[i] = a[i];
    return w;
}

/* W = G' g G'^T, [K][C][4][4] */
void oracle_f2_filter_transform_i16(const int16_t* g, int K, int C, int64_t* out) {
    for (int64_t kc = 0; kc < (int64_t)K * C; ++kc) {
        const int16_t* f = g + kc * 9;
        int64_t u[4][3];
        for (int r = 0; r < 4; ++r)
            for (int c = 0; c < 3; ++c) {
                u[r][c] = 0;
                for (int i = 0; i < 3; ++i) u[r][c] += (int64_t)G2[r][i] * f[i * 3 + c];
            }
        for (int r = 0; r < 4; ++r)
            for (int c = 0; c < 4; ++c) {
                int64_t s = 0;
                for (int j = 0; j < 3; ++j) s += u[r][j] * G2[c][j];
                out[kc * 16 + r * 4 + c] = s;
            }
    }
}

void oracle_f2_filter_transform(const int8_t* g, int K, int C, int64_t* out) {
    int16_t* w = widen(g, (size_t)K * C * 9);
    if (w) oracle_f2_filter_transform_i16(w, K, C, out);
    free(w);
}

/* D = B^T d B for every tile and channel of one batch, [T][C][4][4] */
void oracle_f2_input_transform_i16(const int16_t* x, int N, int C, int H, int W, int64_t* out) {
    int TH = cdiv(H, 2), TW = cdiv(W, 2);
    #pragma omp parallel for collapse(2)
    for (int n = 0; n < N; ++n)
        for (int ty = 0; ty < TH; ++ty)
            for (int tx = 0; tx < TW; ++tx) {
                size_t t = ((size_t)n * TH + ty) * TW + tx;
                for (int c = 0; c < C; ++c) {
                    int64_t d[4][4], u[4][4];
                    for (int a = 0; a < 4; ++a)
                        for (int b = 0; b < 4; ++b) {
                            int h = 2 * ty - 1 + a, w = 2 * tx - 1 + b;
                            d[a][b] = (h >= 0 && h < H && w >= 0 && w < W)
                                          ? x[(((size_t)n * C + c) * H + h) * W + w] : 0;
                        }
                    for (int r = 0; r < 4; ++r)
                        for (int b = 0; b < 4; ++b) {
                            u[r][b] = 0;
                            for (int a = 0; a < 4; ++a) u[r][b] += (int64_t)B2T[r][a] * d[a][b];
                        }
                    for (int r = 0; r < 4; ++r)
                        for (int cc = 0; cc < 4; ++cc) {
                            int64_t s = 0;
                            for (int b = 0; b < 4; ++b) s += u[r][b] * B2T[cc][b];
                            out[(t * C + c) * 16 + r * 4 + cc] = s;
                        }
                }
            }
}

void oracle_f2_input_transform(const int8_t* x, int N, int C, int H, int W, int64_t* out) {
    int16_t* w = widen(x, (size_t)N * C * H * W);
    if (w) oracle_f2_input_transform_i16(w, N, C, H, W, out);
    free(w);
}

/* Section 4.2, steps 1-4, for one 4x4xC Winograd-domain filter per output channel: the
   largest magnitude over the channels at each of the 16 locations decides one factor
   n/2^p per location (none if it is within the range); every channel's weight there is
   multiplied by it, rounding half up.  Wt [K][C][4][4] in place; tab [K][16][4] = (n,p,r,q)
   with the reciprocal r/2^q of the section's last paragraph; mx_out [K][16]. */
void oracle_f2_scale_filters(int64_t* Wt, int K, int C, int64_t range, int32_t* tab, int64_t* mx_out) {
    for (int k = 0; k < K; ++k)
        for (int e = 0; e < 16; ++e) {
            int64_t mx = 0;
            for (int c = 0; c < C; ++c) {
                int64_t a = llabs(Wt[((size_t)k * C + c) * 16 + e]);
                if (a > mx) mx = a;
            }
            int32_t n, p, r, q;
            oracle_scale_factor(mx, range, &n, &p);
            oracle_inverse_factor(n, p, &r, &q);
            if (n != 0)
                for (int c = 0; c < C; ++c) {
                    int64_t* w = Wt + ((size_t)k * C + c) * 16 + e;
                    *w = oracle_scale_round(*w, n, p);
                }
            int32_t* tb = tab + ((size_t)k * 16 + e) * 4;
            tb[0] = n; tb[1] = p; tb[2] = r; tb[3] = q;
            mx_out[(size_t)k * 16 + e] = mx;
        }
}

/* The same steps applied to the activations, which Section 4.1 says the analysis covers as
   well (11-bit B^T d B for int8 data) but which cannot be prepared offline: what an output
   feature map is for the filters, a tile is for the activations.  For every tile and each of
   its 16 X-Y locations the largest magnitude over the channels decides one factor n/2^p (none
   if it is within the range); every channel's value there is multiplied by it, rounding half
   up.  D [T][C][4][4] in place; tab [T][16][4] = (n,p,r,q); mx_out [T][16]. */
void oracle_f2_scale_activations(int64_t* D, int64_t T, int C, int64_t range, int32_t* tab, int64_t* mx_out) {
    for (int64_t t = 0; t < T; ++t)
        for (int e = 0; e < 16; ++e) {
            int64_t mx = 0;
            for (int c = 0; c < C; ++c) {
                int64_t a = llabs(D[((size_t)t * C + c) * 16 + e]);
                if (a > mx) mx = a;
            }
            int32_t n, p, r, q;
            oracle_scale_factor(mx, range, &n, &p);
            oracle_inverse_factor(n, p, &r, &q);
            if (n != 0)
                for (int c = 0; c < C; ++c) {
                    int64_t* d = D + ((size_t)t * C + c) * 16 + e;
                    *d = oracle_scale_round(*d, n, p);
                }
            int32_t* tb = tab + ((size_t)t * 16 + e) * 4;
            tb[0] = n; tb[1] = p; tb[2] = r; tb[3] = q;
            if (mx_out) mx_out[(size_t)t * 16 + e] = mx;
        }
}

/* Whole path.  mode 0: lossless (y equals the direct convolution); mode 1: filters scaled
   into [-range, range], the channel sums multiplied back by r/2^q (round half up) before
   the output transform, and the final A^T M A / 4 rounded half up; mode 2: mode 1 with the
   activations of every tile scaled into the same range too (oracle_f2_scale_activations); a
   channel sum is multiplied back first by the filter's reciprocal, then by the tile's, each
   step rounding half up.
   Returns a bit mask: 2 = a lossless A^T M A was not divisible by 4, 4 = an output did not
   fit int32; -1 when memory runs out. */
int oracle_f2_conv2d_i16(const int16_t* x, const int16_t* g, int32_t* y, int N, int C, int H, int W,
                         int K, int mode, int64_t range) {
    int TH = cdiv(H, 2), TW = cdiv(W, 2);
    int64_t Timg = (int64_t)TH * TW;
    int64_t* Wt = (int64_t*)malloc((size_t)K * C * 16 * sizeof(int64_t));
    int32_t* tab = (int32_t*)malloc((size_t)K * 16 * 4 * sizeof(int32_t));
    int64_t* mx = (int64_t*)malloc((size_t)K * 16 * sizeof(int64_t));
    int64_t* D = (int64_t*)malloc((size_t)Timg * C * 16 * sizeof(int64_t));
    int32_t* atab = (int32_t*)malloc((size_t)Timg * 16 * 4 * sizeof(int32_t));
    int flags = 0;
    if (!Wt || !tab || !mx || !D || !atab) { flags = -1; goto done; }
    oracle_f2_filter_transform_i16(g, K, C, Wt);
    if (mode >= 1) oracle_f2_scale_filters(Wt, K, C, range, tab, mx);
    for (int n = 0; n < N; ++n) {
        oracle_f2_input_transform_i16(x + (size_t)n * C * H * W, 1, C, H, W, D);
        if (mode == 2) oracle_f2_scale_activations(D, Timg, C, range, atab, NULL);
        #pragma omp parallel for reduction(|:flags)
        for (int64_t t = 0; t < Timg; ++t) {
            int ty = (int)(t / TW), tx = (int)(t % TW);
            for (int k = 0; k < K; ++k) {
                int64_t M[4][4], Z[2][4];
                for (int e = 0; e < 16; ++e) {
                    int64_t s = 0;
                    for (int c = 0; c < C; ++c)
                        s += Wt[((size_t)k * C + c) * 16 + e] * D[((size_t)t * C + c) * 16 + e];
                    if (mode >= 1) {
                        const int32_t* tb = tab + ((size_t)k * 16 + e) * 4;
                        if (tb[0] != 0) s = oracle_scale_round(s, tb[2], tb[3]);
                    }
                    if (mode == 2) {
                        const int32_t* ta = atab + ((size_t)t * 16 + e) * 4;
                        if (ta[0] != 0) s = oracle_scale_round(s, ta[2], ta[3]);
                    }
                    M[e / 4][e % 4] = s;
                }
                for (int i = 0; i < 2; ++i)
                    for (int c = 0; c < 4; ++c) {
                        Z[i][c] = 0;
                        for (int r = 0; r < 4; ++r) Z[i][c] += (int64_t)A2T[i][r] * M[r][c];
                    }
                for (int i = 0; i < 2; ++i)
                    for (int j = 0; j < 2; ++j) {
                        int64_t s = 0;
                        for (int c = 0; c < 4; ++c) s += Z[i][c] * A2T[j][c];
                        if (mode == 0 && (s & 3) != 0) flags |= 2;
                        int64_t v = (s + (mode >= 1 ? 2 : 0)) >> 2;   /* arithmetic shift */
                        if (v > INT32_MAX || v < INT32_MIN) flags |= 4;
                        int h = 2 * ty + i, w = 2 * tx + j;
                        if (h < H && w < W) y[(((size_t)n * K + k) * H + h) * W + w] = (int32_t)v;
                    }
            }
        }
    }
done:
    free(Wt); free(tab); free(mx); free(D); free(atab);
    return flags;
}

int oracle_f2_conv2d(const int8_t* x, const int8_t* g, int32_t* y, int N, int C, int H, int W,
                     int K, int mode, int64_t range) {
    int16_t* xw = widen(x, (size_t)N * C * H * W);
    int16_t* gw = widen(g, (size_t)K * C * 9);
    int flags = (xw && gw) ? oracle_f2_conv2d_i16(xw, gw, y, N, C, H, W, K, mode, range) : -1;
    free(xw); free(gw);
    return flags;
}

/* Direct 3x3 stride-1 pad-1 correlation of 16-bit inputs (the definition the int9 path is
   checked against); returns 4 if an output did not fit int32, else 0. */
int oracle_direct_conv2d_i16(const int16_t* x, const int16_t* g, int32_t* y, int N, int C, int H, int W, int K) {
    int flags = 0;
    #pragma omp parallel for collapse(2) reduction(|:flags)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w) {
                    int64_t s = 0;
                    for (int c = 0; c < C; ++c)
                        for (int a = 0; a < 3; ++a)
                            for (int b = 0; b < 3; ++b) {
                                int hh = h + a - 1, ww = w + b - 1;
                                if (hh < 0 || hh >= H || ww < 0 || ww >= W) continue;
                                s += (int64_t)x[(((size_t)n * C + c) * H + hh) * W + ww] *
                                     g[(((size_t)k * C + c) * 3 + a) * 3 + b];
                            }
                    if (s > INT32_MAX || s < INT32_MIN) flags |= 4;
                    y[(((size_t)n * K + k) * H + h) * W + w] = (int32_t)s;
                }
    return flags;
}
