/*
 * CPU ORACLE -- test infrastructure, not product code.
 *
 * A plain, slow, obviously-correct reference for the integer complex Winograd
 * F(4x4,3x3) convolution of Meng & Brothers, "Efficient Winograd Convolution
 * via Integer Arithmetic" (SysML 2019).  Only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code, header, table
 * or helper with the HIP library.
 *
 * Everything is written as the matrix definitions of the paper, with Gaussian
 * integers held as explicit (re, im) int64 pairs and full 6x6 complex tiles:
 * the conjugate symmetry of Section 3.4 is never assumed here, so tests can
 * check it.  No blocking, fusion or reordering.
 *
 * Parity status of each function (what pins it; the pins live in tests/):
 *   oracle_direct_conv2d        pinned: library conv2d in float64, tiny brute force
 *   oracle_input_transform      pinned: printed B^T (golden fixture) via matrix product;
 *                               row expansion of B^T d printed in Section 3.4
 *   oracle_filter_transform     pinned: printed G (golden fixture); 12-bit bound
 *   oracle_contract / oracle_output_transform / oracle_winograd_conv2d (lossless)
 *                               pinned: exact equality with the direct convolution
 *   oracle_worstcase_magnitude  pinned: the 1020/1530/2295 table of Section 4.1
 *   oracle_scale_factor         pinned: Table 1 membership, brute-force maximality,
 *                               the "4-bit n", "p in 4..7" prose of Section 4.2
 *   oracle_inverse_factor       pinned: "8-bit multiply, shift 4..7" of Section 4.2
 *   scaled-mode pipeline        special cases pinned (small weights, huge range
 *                               => equals lossless); the general lossy result is
 *                               PARITY UNPINNED: the paper prints no worked example
 *                               for it, only the 1.12 / 0.1% mean-error statistics
 *                               (used as a weak pin on the rounding mode).
 *   oracle_scale_activations, oracle_inverse_scale_tiles, mode 2 (activations scaled as well)
 *                               Section 4.1 only remarks that the analysis of Section 4.2
 *                               carries over to B^T d B; the rule here is that section's with
 *                               a tile in the place of an output feature map (see the
 *                               function).  Special cases pinned (no tile needs scaling =>
 *                               equals mode 1; scaled activations within the range and
 *                               conjugate-symmetric; table entries from the pinned factor
 *                               routines; a tile's operands do not depend on other tiles; a
 *                               single-tile case followed by hand); the general lossy result
 *                               is PARITY UNPINNED.
 *   *_i16 variants              the same definitions on 16-bit inputs: the quantised tensors of
 *                               Section 4.1 (uint8 minus zero point = int9); lossless pinned by
 *                               exact equality with the 16-bit direct convolution, the int8
 *                               functions on int8 data, and the 16 * 255 = 4080 worst case
 *   oracle_requant_relu_pool    not in the paper (harness glue); pinned by a numpy
 *                               one-liner on small inputs only.
 *
 * Layouts: activations NCHW int8, filters [K][C][3][3] int8, outputs NCHW int32.
 * Tile t = (n*TH + ty)*TW + tx, TH = ceil(H/4), TW = ceil(W/4); tile (ty,tx)
 * reads input rows 4ty-1 .. 4ty+4 and columns 4tx-1 .. 4tx+4 (zero outside the
 * image: pad 1) and owns outputs rows 4ty .. 4ty+3, columns 4tx .. 4tx+3.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct { int64_t re, im; } gint;   /* a Gaussian integer */

static gint gi(int64_t re, int64_t im) { gint z; z.re = re; z.im = im; return z; }
static gint gi_add(gint a, gint b) { return gi(a.re + b.re, a.im + b.im); }
static gint gi_mul(gint a, gint b) {
    /* the plain four-multiplication product; the three-multiplication form of
       Section 3.1 yields the same integers */
    return gi(a.re * b.re - a.im * b.im, a.re * b.im + a.im * b.re);
}
static gint gi_conj(gint a) { return gi(a.re, -a.im); }

/* Section 3.3: the transform matrices of complex F(4x4,3x3), points 0,1,-1,i,-i
   and infinity.  Entries are written {re, im}. */
static const int8_t BT_[6][6][2] = {
    {{1,0},{0, 0},{ 0,0},{ 0, 0},{-1,0},{0,0}},
    {{0,0},{1, 0},{ 1,0},{ 1, 0},{ 1,0},{0,0}},
    {{0,0},{-1,0},{ 1,0},{-1, 0},{ 1,0},{0,0}},
    {{0,0},{0,-1},{-1,0},{ 0, 1},{ 1,0},{0,0}},
    {{0,0},{0, 1},{-1,0},{ 0,-1},{ 1,0},{0,0}},
    {{0,0},{-1,0},{ 0,0},{ 0, 0},{ 0,0},{1,0}},
};
/* G' = 4 G: the filter transform made integral (Section 3.3 gives G with
   denominators 4; Section 4.1 does the same scaling by 2 for F(2x2,3x3)). */
static const int8_t G4_[6][3][2] = {
    {{4,0},{0, 0},{ 0,0}},
    {{1,0},{1, 0},{ 1,0}},
    {{1,0},{-1,0},{ 1,0}},
    {{1,0},{0, 1},{-1,0}},
    {{1,0},{0,-1},{-1,0}},
    {{0,0},{0, 0},{ 4,0}},
};
static const int8_t AT_[4][6][2] = {
    {{1,0},{1,0},{ 1,0},{ 1, 0},{ 1, 0},{0,0}},
    {{0,0},{1,0},{-1,0},{ 0, 1},{ 0,-1},{0,0}},
    {{0,0},{1,0},{ 1,0},{-1, 0},{-1, 0},{0,0}},
    {{0,0},{1,0},{-1,0},{ 0,-1},{ 0, 1},{1,0}},
};
static gint BT(int r, int c) { return gi(BT_[r][c][0], BT_[r][c][1]); }
static gint G4(int r, int c) { return gi(G4_[r][c][0], G4_[r][c][1]); }
static gint AT(int r, int c) { return gi(AT_[r][c][0], AT_[r][c][1]); }

/* Copies of the constants for tests that want to look at them. */
void oracle_get_matrices(int8_t* bt, int8_t* g4, int8_t* at) {
    memcpy(bt, BT_, sizeof BT_);
    memcpy(g4, G4_, sizeof G4_);
    memcpy(at, AT_, sizeof AT_);
}

/* Section 3.4: which entries of a transformed 6x6 tile are the conjugate of
   which.  partner[r][c] = {r', c'} such that X[r][c] = conj(X[r'][c']);
   an entry whose partner is itself is real.  Canonical entries are those with
   no 4 in their index. */
static void partner_of(int r, int c, int* pr, int* pc) {
    int rr = r, cc = c;
    if (r == 4 && c == 4)      { rr = 3; cc = 3; }
    else if (r == 4 && c == 3) { rr = 3; cc = 4; }
    else if (r == 3 && c == 4) { rr = 3; cc = 4; }   /* canonical on its own */
    else if (r == 4)           { rr = 3; }
    else if (c == 4)           { cc = 3; }
    *pr = rr; *pc = cc;
}
static int is_canonical(int r, int c) {
    int pr, pc; partner_of(r, c, &pr, &pc);
    return pr == r && pc == c;
}
void oracle_partner_map(int32_t* out /* [6][6][2] */) {
    for (int r = 0; r < 6; ++r)
        for (int c = 0; c < 6; ++c) {
            int pr, pc; partner_of(r, c, &pr, &pc);
            out[(r * 6 + c) * 2 + 0] = pr;
            out[(r * 6 + c) * 2 + 1] = pc;
        }
}

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

/* ------------------------------------------------------------------------- */
/* Direct convolution: the problem statement (Section 3.2, F(m,r) as an FIR   */
/* filter, nested in two dimensions): y[k] = sum_j g[j] d[k+j], no flip.      */
/* Returns 0, or 1 if some output does not fit int32.                         */
int oracle_direct_conv2d(const int8_t* x, const int8_t* g, int32_t* y,
                         int N, int C, int H, int W, int K) {
    int overflow = 0;
    #pragma omp parallel for collapse(2) reduction(|:overflow)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w) {
                    int64_t acc = 0;
                    for (int c = 0; c < C; ++c)
                        for (int a = 0; a < 3; ++a)
                            for (int b = 0; b < 3; ++b) {
                                int hh = h + a - 1, ww = w + b - 1;
                                if (hh < 0 || hh >= H || ww < 0 || ww >= W) continue;
                                acc += (int64_t)x[(((size_t)n * C + c) * H + hh) * W + ww] *
                                       (int64_t)g[(((size_t)k * C + c) * 3 + a) * 3 + b];
                            }
                    if (acc > INT32_MAX || acc < INT32_MIN) overflow = 1;
                    y[(((size_t)n * K + k) * H + h) * W + w] = (int32_t)acc;
                }
    return overflow;
}

/* ------------------------------------------------------------------------- */
/* Per-tile transforms, written as the matrix products they are.              */

/* D = B^T d B (Section 3.3 / 3.4).  B is the plain transpose of B^T. */
static void tile_input_transform(const int64_t d[6][6], gint D[6][6]) {
    gint tmp[6][6];
    for (int r = 0; r < 6; ++r)
        for (int j = 0; j < 6; ++j) {
            gint s = gi(0, 0);
            for (int a = 0; a < 6; ++a) s = gi_add(s, gi_mul(BT(r, a), gi(d[a][j], 0)));
            tmp[r][j] = s;
        }
    for (int r = 0; r < 6; ++r)
        for (int c = 0; c < 6; ++c) {
            gint s = gi(0, 0);
            for (int j = 0; j < 6; ++j) s = gi_add(s, gi_mul(tmp[r][j], BT(c, j)));
            D[r][c] = s;
        }
}

/* W = G' g G'^T with G' = 4G (Section 3.3), so W is 16x the paper's W. */
static void tile_filter_transform(const int64_t g[3][3], gint Wt[6][6]) {
    gint tmp[6][3];
    for (int r = 0; r < 6; ++r)
        for (int j = 0; j < 3; ++j) {
            gint s = gi(0, 0);
            for (int a = 0; a < 3; ++a) s = gi_add(s, gi_mul(G4(r, a), gi(g[a][j], 0)));
            tmp[r][j] = s;
        }
    for (int r = 0; r < 6; ++r)
        for (int c = 0; c < 6; ++c) {
            gint s = gi(0, 0);
            for (int j = 0; j < 3; ++j) s = gi_add(s, gi_mul(tmp[r][j], G4(c, j)));
            Wt[r][c] = s;
        }
}

/* Y = A^T M A (Section 3.3). */
static void tile_output_transform(const gint M[6][6], gint Y[4][4]) {
    gint tmp[4][6];
    for (int i = 0; i < 4; ++i)
        for (int c = 0; c < 6; ++c) {
            gint s = gi(0, 0);
            for (int r = 0; r < 6; ++r) s = gi_add(s, gi_mul(AT(i, r), M[r][c]));
            tmp[i][c] = s;
        }
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j) {
            gint s = gi(0, 0);
            for (int c = 0; c < 6; ++c) s = gi_add(s, gi_mul(tmp[i][c], AT(j, c)));
            Y[i][j] = s;
        }
}

/* One-dimensional F(4,3): y = A^T [ (G' g) . (B^T d) ], 4 outputs from 6 inputs
   and 3 taps, equal to 4x the FIR result (Section 3.2).  For unit tests. */
void oracle_f43_1d(const int64_t* d /*6*/, const int64_t* g /*3*/, int64_t* y_re /*4*/,
                   int64_t* y_im /*4*/) {
    gint U[6], V[6];
    for (int r = 0; r < 6; ++r) {
        gint s = gi(0, 0), t = gi(0, 0);
        for (int a = 0; a < 3; ++a) s = gi_add(s, gi_mul(G4(r, a), gi(g[a], 0)));
        for (int a = 0; a < 6; ++a) t = gi_add(t, gi_mul(BT(r, a), gi(d[a], 0)));
        U[r] = s; V[r] = t;
    }
    for (int i = 0; i < 4; ++i) {
        gint s = gi(0, 0);
        for (int r = 0; r < 6; ++r) s = gi_add(s, gi_mul(AT(i, r), gi_mul(U[r], V[r])));
        y_re[i] = s.re; y_im[i] = s.im;
    }
}

/* ------------------------------------------------------------------------- */
/* Bulk stages.  A transformed tile is stored as int64 [6][6][2] (re, im).     */

/* D[t][c] = B^T d B for every tile and channel.  out: [T][C][6][6][2]. */
void oracle_input_transform(const int8_t* x, int N, int C, int H, int W, int64_t* out) {
    int TH = ceil_div(H, 4), TW = ceil_div(W, 4);
    #pragma omp parallel for collapse(2)
    for (int n = 0; n < N; ++n)
        for (int ty = 0; ty < TH; ++ty)
            for (int tx = 0; tx < TW; ++tx) {
                size_t t = ((size_t)n * TH + ty) * TW + tx;
                for (int c = 0; c < C; ++c) {
                    int64_t d[6][6];
                    gint D[6][6];
                    for (int a = 0; a < 6; ++a)
                        for (int b = 0; b < 6; ++b) {
                            int hh = 4 * ty - 1 + a, ww = 4 * tx - 1 + b;
                            d[a][b] = (hh < 0 || hh >= H || ww < 0 || ww >= W)
                                          ? 0
                                          : x[(((size_t)n * C + c) * H + hh) * W + ww];
                        }
                    tile_input_transform(d, D);
                    int64_t* o = out + (t * C + c) * 72;
                    for (int r = 0; r < 6; ++r)
                        for (int cc = 0; cc < 6; ++cc) {
                            o[(r * 6 + cc) * 2 + 0] = D[r][cc].re;
                            o[(r * 6 + cc) * 2 + 1] = D[r][cc].im;
                        }
                }
            }
}

/* W[k][c] = G' g G'^T.  out: [K][C][6][6][2]. */
void oracle_filter_transform(const int8_t* g, int K, int C, int64_t* out) {
    #pragma omp parallel for
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < C; ++c) {
            int64_t f[3][3];
            gint Wt[6][6];
            for (int a = 0; a < 3; ++a)
                for (int b = 0; b < 3; ++b) f[a][b] = g[(((size_t)k * C + c) * 3 + a) * 3 + b];
            tile_filter_transform(f, Wt);
            int64_t* o = out + ((size_t)k * C + c) * 72;
            for (int r = 0; r < 6; ++r)
                for (int cc = 0; cc < 6; ++cc) {
                    o[(r * 6 + cc) * 2 + 0] = Wt[r][cc].re;
                    o[(r * 6 + cc) * 2 + 1] = Wt[r][cc].im;
                }
        }
}

/* Winograd-domain accumulation M[t][k] = sum_c W[k][c] (.) D[t][c], the Hadamard
   product of Section 3.4 summed over input channels, at all 36 entries.
   D: [T][C][6][6][2], Wt: [K][C][6][6][2], M: [T][K][6][6][2]. */
void oracle_contract(const int64_t* D, const int64_t* Wt, int64_t T, int C, int K, int64_t* M) {
    #pragma omp parallel for collapse(2)
    for (int64_t t = 0; t < T; ++t)
        for (int k = 0; k < K; ++k) {
            gint acc[36];
            for (int e = 0; e < 36; ++e) acc[e] = gi(0, 0);
            for (int c = 0; c < C; ++c) {
                const int64_t* d = D + ((size_t)t * C + c) * 72;
                const int64_t* w = Wt + ((size_t)k * C + c) * 72;
                for (int e = 0; e < 36; ++e)
                    acc[e] = gi_add(acc[e], gi_mul(gi(w[2 * e], w[2 * e + 1]),
                                                   gi(d[2 * e], d[2 * e + 1])));
            }
            int64_t* m = M + ((size_t)t * K + k) * 72;
            for (int e = 0; e < 36; ++e) { m[2 * e] = acc[e].re; m[2 * e + 1] = acc[e].im; }
        }
}

/* y = (A^T M A + round) >> shift for every tile, stored NCHW int32, clipped to
   the image for partial tiles.  shift = 4 and round = 0 in the lossless path
   (A^T M A is exactly 16 y there), round = 8 in the scaled path.
   Returns a bit mask: 1 = some imaginary part of A^T M A was not zero
   (Section 3.4 says they vanish), 2 = some value was not divisible by 2^shift
   while round == 0, 4 = some output did not fit int32. */
int oracle_output_transform(const int64_t* M, int N, int K, int H, int W, int shift,
                            int64_t round, int32_t* y) {
    int TH = ceil_div(H, 4), TW = ceil_div(W, 4);
    int flags = 0;
    #pragma omp parallel for collapse(2) reduction(|:flags)
    for (int n = 0; n < N; ++n)
        for (int ty = 0; ty < TH; ++ty)
            for (int tx = 0; tx < TW; ++tx) {
                size_t t = ((size_t)n * TH + ty) * TW + tx;
                for (int k = 0; k < K; ++k) {
                    const int64_t* m = M + (t * K + k) * 72;
                    gint Mt[6][6], Y[4][4];
                    for (int r = 0; r < 6; ++r)
                        for (int c = 0; c < 6; ++c)
                            Mt[r][c] = gi(m[(r * 6 + c) * 2], m[(r * 6 + c) * 2 + 1]);
                    tile_output_transform(Mt, Y);
                    for (int i = 0; i < 4; ++i)
                        for (int j = 0; j < 4; ++j) {
                            int h = 4 * ty + i, w = 4 * tx + j;
                            if (Y[i][j].im != 0) flags |= 1;
                            if (round == 0 && (Y[i][j].re & (((int64_t)1 << shift) - 1)) != 0)
                                flags |= 2;
                            int64_t v = (Y[i][j].re + round) >> shift;   /* arithmetic shift */
                            if (v > INT32_MAX || v < INT32_MIN) flags |= 4;
                            if (h < H && w < W)
                                y[(((size_t)n * K + k) * H + h) * W + w] = (int32_t)v;
                        }
                }
            }
    return flags;
}

/* ------------------------------------------------------------------------- */
/* Bit-width analysis (Section 4.1): the worst-case magnitude of every entry  */
/* of G' g G'^T when each filter tap lies in [-gneg, gpos].  G' is any         */
/* rows x 3 Gaussian-integer matrix, given as int [rows][3][2].  The real and  */
/* imaginary parts are each a signed sum of taps; the worst case drives every  */
/* tap to the end of its range that matches the sign of its coefficient.       */
void oracle_worstcase_magnitude(const int32_t* Gm, int rows, int64_t gpos, int64_t gneg,
                                int64_t* out_re /*[rows][rows]*/, int64_t* out_im) {
    for (int r = 0; r < rows; ++r)
        for (int c = 0; c < rows; ++c) {
            int64_t pos_re = 0, neg_re = 0, pos_im = 0, neg_im = 0;
            for (int a = 0; a < 3; ++a)
                for (int b = 0; b < 3; ++b) {
                    gint coef = gi_mul(gi(Gm[(r * 3 + a) * 2], Gm[(r * 3 + a) * 2 + 1]),
                                       gi(Gm[(c * 3 + b) * 2], Gm[(c * 3 + b) * 2 + 1]));
                    if (coef.re > 0) pos_re += coef.re; else neg_re -= coef.re;
                    if (coef.im > 0) pos_im += coef.im; else neg_im -= coef.im;
                }
            /* largest value: positive coefficients at +gpos, negative at -gneg;
               smallest value: the other way round */
            int64_t hi_re = pos_re * gpos + neg_re * gneg, lo_re = pos_re * gneg + neg_re * gpos;
            int64_t hi_im = pos_im * gpos + neg_im * gneg, lo_im = pos_im * gneg + neg_im * gpos;
            out_re[r * rows + c] = hi_re > lo_re ? hi_re : lo_re;
            out_im[r * rows + c] = hi_im > lo_im ? hi_im : lo_im;
        }
}

/* The same analysis for B^T d B with every activation in [-dneg, dpos]. */
void oracle_worstcase_input_magnitude(int64_t dpos, int64_t dneg, int64_t* out_re /*[6][6]*/,
                                      int64_t* out_im) {
    for (int r = 0; r < 6; ++r)
        for (int c = 0; c < 6; ++c) {
            int64_t pos_re = 0, neg_re = 0, pos_im = 0, neg_im = 0;
            for (int a = 0; a < 6; ++a)
                for (int b = 0; b < 6; ++b) {
                    gint coef = gi_mul(BT(r, a), BT(c, b));
                    if (coef.re > 0) pos_re += coef.re; else neg_re -= coef.re;
                    if (coef.im > 0) pos_im += coef.im; else neg_im -= coef.im;
                }
            int64_t hi_re = pos_re * dpos + neg_re * dneg, lo_re = pos_re * dneg + neg_re * dpos;
            int64_t hi_im = pos_im * dpos + neg_im * dneg, lo_im = pos_im * dneg + neg_im * dpos;
            out_re[r * 6 + c] = hi_re > lo_re ? hi_re : lo_re;
            out_im[r * 6 + c] = hi_im > lo_im ? hi_im : lo_im;
        }
}

/* ------------------------------------------------------------------------- */
/* Filter precision scaling (Section 4.2).                                     */

/* Down-scale factor n / 2^p for a location whose largest magnitude over the
   input channels is mx, with spatial weight range [-range, range].
   mx <= range: n = p = 0, "no scaling".  Otherwise the largest n / 2^p with a
   4-bit n (n in 8..15 once normalised) such that n*mx <= range * 2^p:
       x = range*128 / mx,  y = floor(log2 x),  n = floor(x / 2^(y-3)),  p = 10 - y
   done in exact integer arithmetic.  (The printed steps divide by 2^(y-4) and
   set p = 7-(y-4); that yields a 5-bit n and p = 8 for the paper's own maximum
   2295, against its "4-bit n", "p from 4 to 7" and Table 1.  Using y-3 agrees
   with all three.) */
void oracle_scale_factor(int64_t mx, int64_t range, int32_t* n_out, int32_t* p_out) {
    if (mx <= range) { *n_out = 0; *p_out = 0; return; }
    /* y = floor(log2(range*128/mx)): the largest y with mx * 2^y <= range*128.
       y may be negative when mx > range*128; handle by scaling the other side. */
    int y = 0;
    int64_t num = range * 128;
    if (mx <= num) { while ((mx << (y + 1)) <= num) ++y; }
    else           { while (mx > (num << (-y))) --y; }
    /* n = floor( x / 2^(y-3) ) = floor( num * 8 / (mx * 2^y) ) */
    int64_t n = (y >= 0) ? (num * 8) / (mx << y) : ((num * 8) << (-y)) / mx;
    *n_out = (int32_t)n;
    *p_out = 10 - y;
}

/* Integer approximation of the reciprocal 2^p / n as r / 2^q: an 8-bit r and
   the largest q in 0..7 that keeps r = floor(2^(p+q)/n + 1/2) <= 255. */
void oracle_inverse_factor(int32_t n, int32_t p, int32_t* r_out, int32_t* q_out) {
    if (n == 0) { *r_out = 1; *q_out = 0; return; }
    for (int q = 7; q >= 0; --q) {
        int64_t r = ((((int64_t)1 << (p + q)) * 2) + n) / (2 * (int64_t)n);  /* round half up */
        if (r <= 255) { *r_out = (int32_t)r; *q_out = q; return; }
    }
    *r_out = 0; *q_out = -1;   /* not representable: 2^p / n > 255 */
}

/* round-half-up scaling of one integer: (v*mul + 2^(sh-1)) >> sh, arithmetic shift */
static int64_t scale_round(int64_t v, int64_t mul, int sh) {
    int64_t prod = v * mul;
    if (sh == 0) return prod;
    return (prod + ((int64_t)1 << (sh - 1))) >> sh;
}
int64_t oracle_scale_round(int64_t v, int64_t mul, int sh) { return scale_round(v, mul, sh); }

/* Steps 1-4 and the down-scaling of Section 4.2 for complex F(4x4,3x3):
   one factor per output channel k and canonical location, from the largest
   max(|Re|,|Im|) over the input channels; the factor multiplies Re and Im of
   every channel's weight at that location (round half up); the conjugate
   partner locations are then the conjugates of the scaled canonical ones.
   Wt: [K][C][6][6][2] in place.  tab: [K][6][6][4] = (n, p, r, q) at every
   location (partners repeat their canonical entry).  mx_out: [K][6][6]. */
void oracle_scale_filters(int64_t* Wt, int K, int C, int64_t range, int32_t* tab,
                          int64_t* mx_out) {
    for (int k = 0; k < K; ++k) {
        for (int r = 0; r < 6; ++r)
            for (int c = 0; c < 6; ++c) {
                if (!is_canonical(r, c)) continue;
                int e = r * 6 + c;
                int64_t mx = 0;
                for (int ch = 0; ch < C; ++ch) {
                    const int64_t* w = Wt + ((size_t)k * C + ch) * 72;
                    int64_t a = llabs(w[2 * e]), b = llabs(w[2 * e + 1]);
                    if (a > mx) mx = a;
                    if (b > mx) mx = b;
                }
                int32_t n, p, rr, q;
                oracle_scale_factor(mx, range, &n, &p);
                oracle_inverse_factor(n, p, &rr, &q);
                if (n != 0)
                    for (int ch = 0; ch < C; ++ch) {
                        int64_t* w = Wt + ((size_t)k * C + ch) * 72;
                        w[2 * e]     = scale_round(w[2 * e], n, p);
                        w[2 * e + 1] = scale_round(w[2 * e + 1], n, p);
                    }
                int32_t* tb = tab + ((size_t)k * 36 + e) * 4;
                tb[0] = n; tb[1] = p; tb[2] = rr; tb[3] = q;
                mx_out[(size_t)k * 36 + e] = mx;
            }
        for (int r = 0; r < 6; ++r)
            for (int c = 0; c < 6; ++c) {
                if (is_canonical(r, c)) continue;
                int pr, pc; partner_of(r, c, &pr, &pc);
                int e = r * 6 + c, pe = pr * 6 + pc;
                for (int ch = 0; ch < C; ++ch) {
                    int64_t* w = Wt + ((size_t)k * C + ch) * 72;
                    w[2 * e] = w[2 * pe];
                    w[2 * e + 1] = -w[2 * pe + 1];
                }
                memcpy(tab + ((size_t)k * 36 + e) * 4, tab + ((size_t)k * 36 + pe) * 4,
                       4 * sizeof(int32_t));
                mx_out[(size_t)k * 36 + e] = mx_out[(size_t)k * 36 + pe];
            }
    }
}

/* Reverse scaling before the output transform (Section 4.2): at each canonical
   location M = (M~ * r + 2^(q-1)) >> q on Re and Im separately; partner
   locations become the conjugates of the result.  M: [T][K][6][6][2] in place. */
void oracle_inverse_scale(int64_t* M, int64_t T, int K, const int32_t* tab) {
    #pragma omp parallel for
    for (int64_t t = 0; t < T; ++t)
        for (int k = 0; k < K; ++k) {
            int64_t* m = M + ((size_t)t * K + k) * 72;
            for (int r = 0; r < 6; ++r)
                for (int c = 0; c < 6; ++c) {
                    if (!is_canonical(r, c)) continue;
                    int e = r * 6 + c;
                    const int32_t* tb = tab + ((size_t)k * 36 + e) * 4;
                    if (tb[0] == 0) continue;
                    m[2 * e]     = scale_round(m[2 * e], tb[2], tb[3]);
                    m[2 * e + 1] = scale_round(m[2 * e + 1], tb[2], tb[3]);
                }
            for (int r = 0; r < 6; ++r)
                for (int c = 0; c < 6; ++c) {
                    if (is_canonical(r, c)) continue;
                    int pr, pc; partner_of(r, c, &pr, &pc);
                    gint z = gi_conj(gi(m[2 * (pr * 6 + pc)], m[2 * (pr * 6 + pc) + 1]));
                    m[2 * (r * 6 + c)] = z.re;
                    m[2 * (r * 6 + c) + 1] = z.im;
                }
        }
}

/* The remark that closes Section 4.1: the analysis of Section 4.2 applies to the
   transformed activations B^T d B as well (12 bits here for int8 data), although
   they cannot be prepared offline.  The rule below is Section 4.2's with a tile in
   the place of an output feature map: for every tile and canonical location the
   largest max(|Re|,|Im|) over the input channels decides one factor n/2^p (none if
   it is within the range); Re and Im of every channel's value there are multiplied
   by it, rounding half up; partner locations become the conjugates of the scaled
   canonical ones.  D: [T][C][6][6][2] in place.  tab: [T][6][6][4] = (n, p, r, q)
   at every location (partners repeat their canonical entry).  mx_out (may be NULL):
   [T][6][6]. */
void oracle_scale_activations(int64_t* D, int64_t T, int C, int64_t range, int32_t* tab,
                              int64_t* mx_out) {
    for (int64_t t = 0; t < T; ++t) {
        for (int r = 0; r < 6; ++r)
            for (int c = 0; c < 6; ++c) {
                if (!is_canonical(r, c)) continue;
                int e = r * 6 + c;
                int64_t mx = 0;
                for (int ch = 0; ch < C; ++ch) {
                    const int64_t* d = D + ((size_t)t * C + ch) * 72;
                    int64_t a = llabs(d[2 * e]), b = llabs(d[2 * e + 1]);
                    if (a > mx) mx = a;
                    if (b > mx) mx = b;
                }
                int32_t n, p, rr, q;
                oracle_scale_factor(mx, range, &n, &p);
                oracle_inverse_factor(n, p, &rr, &q);
                if (n != 0)
                    for (int ch = 0; ch < C; ++ch) {
                        int64_t* d = D + ((size_t)t * C + ch) * 72;
                        d[2 * e]     = scale_round(d[2 * e], n, p);
                        d[2 * e + 1] = scale_round(d[2 * e + 1], n, p);
                    }
                int32_t* tb = tab + ((size_t)t * 36 + e) * 4;
                tb[0] = n; tb[1] = p; tb[2] = rr; tb[3] = q;
                if (mx_out) mx_out[(size_t)t * 36 + e] = mx;
            }
        for (int r = 0; r < 6; ++r)
            for (int c = 0; c < 6; ++c) {
                if (is_canonical(r, c)) continue;
                int pr, pc; partner_of(r, c, &pr, &pc);
                int e = r * 6 + c, pe = pr * 6 + pc;
                for (int ch = 0; ch < C; ++ch) {
                    int64_t* d = D + ((size_t)t * C + ch) * 72;
                    d[2 * e] = d[2 * pe];
                    d[2 * e + 1] = -d[2 * pe + 1];
                }
                memcpy(tab + ((size_t)t * 36 + e) * 4, tab + ((size_t)t * 36 + pe) * 4,
                       4 * sizeof(int32_t));
                if (mx_out) mx_out[(size_t)t * 36 + e] = mx_out[(size_t)t * 36 + pe];
            }
    }
}

/* The tile-side reverse scaling: oracle_inverse_scale with the table of the tile
   instead of the filter's.  M: [T][K][6][6][2] in place, atab: [T][6][6][4]. */
void oracle_inverse_scale_tiles(int64_t* M, int64_t T, int K, const int32_t* atab) {
    #pragma omp parallel for
    for (int64_t t = 0; t < T; ++t)
        for (int k = 0; k < K; ++k) {
            int64_t* m = M + ((size_t)t * K + k) * 72;
            for (int r = 0; r < 6; ++r)
                for (int c = 0; c < 6; ++c) {
                    if (!is_canonical(r, c)) continue;
                    int e = r * 6 + c;
                    const int32_t* tb = atab + ((size_t)t * 36 + e) * 4;
                    if (tb[0] == 0) continue;
                    m[2 * e]     = scale_round(m[2 * e], tb[2], tb[3]);
                    m[2 * e + 1] = scale_round(m[2 * e + 1], tb[2], tb[3]);
                }
            for (int r = 0; r < 6; ++r)
                for (int c = 0; c < 6; ++c) {
                    if (is_canonical(r, c)) continue;
                    int pr, pc; partner_of(r, c, &pr, &pc);
                    gint z = gi_conj(gi(m[2 * (pr * 6 + pc)], m[2 * (pr * 6 + pc) + 1]));
                    m[2 * (r * 6 + c)] = z.re;
                    m[2 * (r * 6 + c) + 1] = z.im;
                }
        }
}

/* ------------------------------------------------------------------------- */
/* Whole path, one image at a time so memory stays bounded.                    */
/* mode 0: lossless, y must equal the direct convolution bit for bit.          */
/* mode 1: filter-scaled with weight range [-range, range].                    */
/* mode 2: mode 1 with the activations of every tile scaled into the same      */
/*         range too (oracle_scale_activations); a channel sum is multiplied   */
/*         back first by the filter's reciprocal, then by the tile's, each     */
/*         step rounding half up.                                              */
/* Returns the OR of oracle_output_transform's flags over the images, or -1    */
/* when memory runs out.                                                       */
int oracle_winograd_conv2d(const int8_t* x, const int8_t* g, int32_t* y, int N, int C, int H,
                           int W, int K, int mode, int64_t range) {
    int TH = ceil_div(H, 4), TW = ceil_div(W, 4);
    int64_t Timg = (int64_t)TH * TW;
    int64_t* Wt = (int64_t*)malloc((size_t)K * C * 72 * sizeof(int64_t));
    int32_t* tab = (int32_t*)malloc((size_t)K * 36 * 4 * sizeof(int32_t));
    int64_t* mx = (int64_t*)malloc((size_t)K * 36 * sizeof(int64_t));
    int64_t* D = (int64_t*)malloc((size_t)Timg * C * 72 * sizeof(int64_t));
    int64_t* M = (int64_t*)malloc((size_t)Timg * K * 72 * sizeof(int64_t));
    int32_t* atab = (int32_t*)malloc((size_t)Timg * 36 * 4 * sizeof(int32_t));
    int flags = 0;
    if (!Wt || !tab || !mx || !D || !M || !atab) { flags = -1; goto done; }
    oracle_filter_transform(g, K, C, Wt);
    if (mode >= 1) oracle_scale_filters(Wt, K, C, range, tab, mx);
    for (int n = 0; n < N; ++n) {
        oracle_input_transform(x + (size_t)n * C * H * W, 1, C, H, W, D);
        if (mode == 2) oracle_scale_activations(D, Timg, C, range, atab, NULL);
        oracle_contract(D, Wt, Timg, C, K, M);
        if (mode >= 1) oracle_inverse_scale(M, Timg, K, tab);
        if (mode == 2) oracle_inverse_scale_tiles(M, Timg, K, atab);
        flags |= oracle_output_transform(M, 1, K, H, W, 4, mode >= 1 ? 8 : 0,
                                         y + (size_t)n * K * H * W);
    }
done:
    free(Wt); free(tab); free(mx); free(D); free(M); free(atab);
    return flags;
}

/* ------------------------------------------------------------------------- */
/* Section 4.1's data model: tensors quantised to uint8 with a zero point are    */
/* the integers byte - zero_point in [-255, 255] (int9), carried here as int16.  */
/* The same definitions as above, written out again for 16-bit inputs.           */

void oracle_input_transform_i16(const int16_t* x, int N, int C, int H, int W, int64_t* out) {
    int TH = ceil_div(H, 4), TW = ceil_div(W, 4);
    #pragma omp parallel for collapse(2)
    for (int n = 0; n < N; ++n)
        for (int ty = 0; ty < TH; ++ty)
            for (int tx = 0; tx < TW; ++tx) {
                size_t t = ((size_t)n * TH + ty) * TW + tx;
                for (int c = 0; c < C; ++c) {
                    int64_t d[6][6];
                    gint D[6][6];
                    for (int a = 0; a < 6; ++a)
                        for (int b = 0; b < 6; ++b) {
                            int hh = 4 * ty - 1 + a, ww = 4 * tx - 1 + b;
                            d[a][b] = (hh < 0 || hh >= H || ww < 0 || ww >= W)
                                          ? 0
                                          : x[(((size_t)n * C + c) * H + hh) * W + ww];
                        }
                    tile_input_transform(d, D);
                    int64_t* o = out + (t * C + c) * 72;
                    for (int r = 0; r < 6; ++r)
                        for (int cc = 0; cc < 6; ++cc) {
                            o[(r * 6 + cc) * 2 + 0] = D[r][cc].re;
                            o[(r * 6 + cc) * 2 + 1] = D[r][cc].im;
                        }
                }
            }
}

void oracle_filter_transform_i16(const int16_t* g, int K, int C, int64_t* out) {
    #pragma omp parallel for
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < C; ++c) {
            int64_t f[3][3];
            gint Wt[6][6];
            for (int a = 0; a < 3; ++a)
                for (int b = 0; b < 3; ++b) f[a][b] = g[(((size_t)k * C + c) * 3 + a) * 3 + b];
            tile_filter_transform(f, Wt);
            int64_t* o = out + ((size_t)k * C + c) * 72;
            for (int r = 0; r < 6; ++r)
                for (int cc = 0; cc < 6; ++cc) {
                    o[(r * 6 + cc) * 2 + 0] = Wt[r][cc].re;
                    o[(r * 6 + cc) * 2 + 1] = Wt[r][cc].im;
                }
        }
}

/* Whole path on 16-bit inputs; modes, range and return value as oracle_winograd_conv2d
   (flag 4: an output did not fit int32, which int9 data can reach from 230 channels on). */
int oracle_winograd_conv2d_i16(const int16_t* x, const int16_t* g, int32_t* y, int N, int C, int H,
                               int W, int K, int mode, int64_t range) {
    int TH = ceil_div(H, 4), TW = ceil_div(W, 4);
    int64_t Timg = (int64_t)TH * TW;
    int64_t* Wt = (int64_t*)malloc((size_t)K * C * 72 * sizeof(int64_t));
    int32_t* tab = (int32_t*)malloc((size_t)K * 36 * 4 * sizeof(int32_t));
    int64_t* mx = (int64_t*)malloc((size_t)K * 36 * sizeof(int64_t));
    int64_t* D = (int64_t*)malloc((size_t)Timg * C * 72 * sizeof(int64_t));
    int64_t* M = (int64_t*)malloc((size_t)Timg * K * 72 * sizeof(int64_t));
    int flags = 0;
    if (!Wt || !tab || !mx || !D || !M) { flags = -1; goto done; }
    oracle_filter_transform_i16(g, K, C, Wt);
    if (mode == 1) oracle_scale_filters(Wt, K, C, range, tab, mx);
    for (int n = 0; n < N; ++n) {
        oracle_input_transform_i16(x + (size_t)n * C * H * W, 1, C, H, W, D);
        oracle_contract(D, Wt, Timg, C, K, M);
        if (mode == 1) oracle_inverse_scale(M, Timg, K, tab);
        flags |= oracle_output_transform(M, 1, K, H, W, 4, mode == 1 ? 8 : 0,
                                         y + (size_t)n * K * H * W);
    }
done:
    free(Wt); free(tab); free(mx); free(D); free(M);
    return flags;
}

/* ------------------------------------------------------------------------- */
/* Harness glue for layer stacks (not in the paper beyond the remark that a    */
/* requantisation follows each quantised convolution, Section 4.4):            */
/* v = (y + 2^(s-1)) >> s (s = 0: v = y), clamp to [lo, 127] with lo = 0 when   */
/* relu else -128, then an optional 2x2 stride-2 max-pool (H, W even).          */
void oracle_requant_relu_pool(const int32_t* y, int8_t* out, int N, int K, int H, int W,
                              int shift, int relu, int pool) {
    int lo = relu ? 0 : -128;
    int Ho = pool ? H / 2 : H, Wo = pool ? W / 2 : W;
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int h = 0; h < Ho; ++h)
                for (int w = 0; w < Wo; ++w) {
                    int best = -129;
                    int span = pool ? 2 : 1;
                    for (int a = 0; a < span; ++a)
                        for (int b = 0; b < span; ++b) {
                            int hh = pool ? 2 * h + a : h, ww = pool ? 2 * w + b : w;
                            int64_t v = y[(((size_t)n * K + k) * H + hh) * W + ww];
                            if (shift > 0) v = (v + ((int64_t)1 << (shift - 1))) >> shift;
                            if (v < lo) v = lo;
                            if (v > 127) v = 127;
                            if (v > best) best = (int)v;
                        }
                    out[(((size_t)n * K + k) * Ho + h) * Wo + w] = (int8_t)best;
                }
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
