/*
 * CPU ORACLE -- test infrastructure, not product code.
 *
 * Drives every function of the oracle on small ragged shapes; built together with the oracle's
 * sources under -fsanitize=address,undefined (tests/test_oracle_sanitize.py), so that an access
 * out of bounds, a signed overflow or a shift out of range anywhere in the oracle aborts the run.
 * It also re-checks two exact identities along the way (lossless Winograd == direct convolution),
 * so a clean exit means more than "did not crash".  Prints "ok" and returns 0.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_direct_conv2d(const int8_t*, const int8_t*, int32_t*, int, int, int, int, int);
int oracle_direct_conv2d_i16(const int16_t*, const int16_t*, int32_t*, int, int, int, int, int);
int oracle_winograd_conv2d(const int8_t*, const int8_t*, int32_t*, int, int, int, int, int, int, int64_t);
int oracle_winograd_conv2d_i16(const int16_t*, const int16_t*, int32_t*, int, int, int, int, int, int, int64_t);
int oracle_f2_conv2d(const int8_t*, const int8_t*, int32_t*, int, int, int, int, int, int, int64_t);
int oracle_f2_conv2d_i16(const int16_t*, const int16_t*, int32_t*, int, int, int, int, int, int, int64_t);
void oracle_requant_relu_pool(const int32_t*, int8_t*, int, int, int, int, int, int, int);
void oracle_worstcase_magnitude(const int32_t*, int, int64_t, int64_t, int64_t*, int64_t*);
void oracle_worstcase_input_magnitude(int64_t, int64_t, int64_t*, int64_t*);
void oracle_scale_factor(int64_t, int64_t, int32_t*, int32_t*);
void oracle_inverse_factor(int32_t, int32_t, int32_t*, int32_t*);
void oracle_f43_1d(const int64_t*, const int64_t*, int64_t*, int64_t*);
void oracle_get_matrices(int8_t*, int8_t*, int8_t*);
void oracle_partner_map(int32_t*);

static uint64_t state = 190101965u;
static int next(int lo, int hi) {   /* splitmix64 */
    uint64_t z = (state += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    z ^= z >> 31;
    return lo + (int)(z % (uint64_t)(hi - lo + 1));
}
static void fail(const char* what) { fprintf(stderr, "sanitize_check: %s\n", what); exit(1); }

static void one_shape(int N, int C, int K, int H, int W, int extremes) {
    size_t nx = (size_t)N * C * H * W, ng = (size_t)K * C * 9, ny = (size_t)N * K * H * W;
    int8_t* x = malloc(nx); int8_t* g = malloc(ng);
    int16_t* x16 = malloc(2 * nx); int16_t* g16 = malloc(2 * ng);
    int32_t* y = malloc(4 * ny); int32_t* w = malloc(4 * ny);
    int8_t* q = malloc(ny);
    if (!x || !g || !x16 || !g16 || !y || !w || !q) fail("out of memory");
    for (size_t i = 0; i < nx; ++i) { x[i] = (int8_t)(extremes ? (next(0, 1) ? 127 : -128) : next(-128, 127)); x16[i] = (int16_t)(extremes ? (next(0, 1) ? 255 : -255) : next(-255, 255)); }
    for (size_t i = 0; i < ng; ++i) { g[i] = (int8_t)(extremes ? (next(0, 1) ? 127 : -128) : next(-128, 127)); g16[i] = (int16_t)(extremes ? (next(0, 1) ? 255 : -255) : next(-255, 255)); }

    if (oracle_direct_conv2d(x, g, y, N, C, H, W, K)) fail("direct convolution overflowed");
    if (oracle_winograd_conv2d(x, g, w, N, C, H, W, K, 0, 127) != 0) fail("lossless F(4x4,3x3) raised a flag");
    if (memcmp(y, w, 4 * ny)) fail("lossless F(4x4,3x3) != direct");
    if (oracle_winograd_conv2d(x, g, w, N, C, H, W, K, 1, 127) & 5) fail("scaled F(4x4,3x3) raised a flag");
    if (oracle_winograd_conv2d(x, g, w, N, C, H, W, K, 2, 127) & 5) fail("F(4x4,3x3) with scaled activations raised a flag");
    if (oracle_f2_conv2d(x, g, w, N, C, H, W, K, 0, 127) & 5) fail("lossless F(2x2,3x3) raised a flag");
    if (memcmp(y, w, 4 * ny)) fail("lossless F(2x2,3x3) != direct");
    if (oracle_f2_conv2d(x, g, w, N, C, H, W, K, 1, 127) & 5) fail("scaled F(2x2,3x3) raised a flag");
    if (oracle_f2_conv2d(x, g, w, N, C, H, W, K, 2, 127) & 5) fail("F(2x2,3x3) with scaled activations raised a flag");
    for (int shift = 0; shift <= 31; shift += 7)
        for (int pool = 0; pool <= ((H % 2 == 0 && W % 2 == 0) ? 1 : 0); ++pool)
            oracle_requant_relu_pool(y, q, N, K, H, W, shift, shift & 1, pool);

    if (oracle_direct_conv2d_i16(x16, g16, y, N, C, H, W, K)) fail("int9 direct convolution overflowed");
    if (oracle_winograd_conv2d_i16(x16, g16, w, N, C, H, W, K, 0, 127) != 0) fail("lossless int9 F(4x4,3x3) raised a flag");
    if (memcmp(y, w, 4 * ny)) fail("lossless int9 F(4x4,3x3) != direct");
    if (oracle_winograd_conv2d_i16(x16, g16, w, N, C, H, W, K, 1, 127) & 5) fail("scaled int9 F(4x4,3x3) raised a flag");
    if (oracle_winograd_conv2d_i16(x16, g16, w, N, C, H, W, K, 1, 255) & 5) fail("scaled int9 F(4x4,3x3), range 255, raised a flag");
    if (oracle_f2_conv2d_i16(x16, g16, w, N, C, H, W, K, 0, 255) & 5) fail("lossless int9 F(2x2,3x3) raised a flag");
    if (memcmp(y, w, 4 * ny)) fail("lossless int9 F(2x2,3x3) != direct");
    if (oracle_f2_conv2d_i16(x16, g16, w, N, C, H, W, K, 1, 255) & 5) fail("scaled int9 F(2x2,3x3) raised a flag");
    free(x); free(g); free(x16); free(g16); free(y); free(w); free(q);
}

int main(void) {
    int8_t bt[72], g4[36], at[48];
    int32_t partner[72];
    oracle_get_matrices(bt, g4, at);
    oracle_partner_map(partner);
    int32_t gm[36];
    for (int i = 0; i < 36; ++i) gm[i] = g4[i];
    int64_t re[36], im[36];
    oracle_worstcase_magnitude(gm, 6, 127, 128, re, im);
    if (re[0] != 16 * 128) fail("worst case of the corner entry");
    oracle_worstcase_magnitude(gm, 6, 255, 255, re, im);
    if (re[0] != 16 * 255) fail("int9 worst case of the corner entry");
    oracle_worstcase_input_magnitude(127, 128, re, im);
    for (int64_t mx = 1; mx <= 5000; ++mx)
        for (int64_t range = 127; range <= 255; range += 128) {
            int32_t n, p, r, q;
            oracle_scale_factor(mx, range, &n, &p);
            oracle_inverse_factor(n, p, &r, &q);
            if (mx > range && (n < 8 || n > 15)) fail("scale factor numerator");
        }
    int64_t d[6] = {1, -2, 3, -4, 5, -6}, g[3] = {7, -8, 9}, yr[4], yi[4];
    oracle_f43_1d(d, g, yr, yi);
    static const int shapes[][5] = {{1, 1, 1, 1, 1}, {1, 3, 2, 5, 7}, {2, 5, 3, 4, 4}, {1, 2, 4, 9, 6}, {1, 7, 2, 13, 3}, {3, 1, 1, 2, 10}};
    for (unsigned i = 0; i < sizeof shapes / sizeof shapes[0]; ++i)
        for (int extremes = 0; extremes <= 1; ++extremes)
            one_shape(shapes[i][0], shapes[i][1], shapes[i][2], shapes[i][3], shapes[i][4], extremes);
    puts("ok");
    return 0;
}
