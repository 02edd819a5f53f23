// The arithmetic of the input transform D = B^T d B (Section 3.3) on the 26 free
// entries (Section 3.4), shared by the stand-alone transform kernel and the
// fused convolution kernel.  Four channels are processed at a time in packed
// 16-bit lanes; `Writer` decides where each int8 operand plane goes.
#pragma once
#include "wg_internal.h"

namespace wg {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef signed char s8x4 __attribute__((ext_vector_type(4)));

// The 6x6 input patch of one tile, four consecutive channels c0..c0+3 per pixel, zero outside
// the image (pad 1) and beyond C.  All loads are issued before any is used: addresses are
// clamped into the image and out-of-range pixels are zeroed afterwards, so no load sits
// behind a branch.
// VEC4 (channels-last input whose C is a multiple of four, chosen on the host): one 4-byte
// load per pixel; a channel group is then either wholly inside or wholly beyond C.
template <int LAYOUT, bool VEC4>
__device__ inline void load_patch(const int8_t* __restrict__ x, const Problem& p, int n, int ty, int tx, int c0,
                                  s16x4 d[6][6]) {
    const int h0 = 4 * ty - 1, w0 = 4 * tx - 1;
    if constexpr (VEC4) {
        static_assert(LAYOUT == WG_NHWC, "4-byte pixel loads need channels-last input");
        const bool have = c0 < p.C;
        s8x4 raw[6][6];
        const int8_t* img = x + (size_t)n * p.H * p.W * p.C + (have ? c0 : 0);
#pragma unroll
        for (int a = 0; a < 6; ++a) {
            const int h = min(max(h0 + a, 0), p.H - 1);
#pragma unroll
            for (int b = 0; b < 6; ++b) {
                const int w = min(max(w0 + b, 0), p.W - 1);
                raw[a][b] = *reinterpret_cast<const s8x4*>(img + ((size_t)h * p.W + w) * p.C);
            }
        }
#pragma unroll
        for (int a = 0; a < 6; ++a)
#pragma unroll
            for (int b = 0; b < 6; ++b) {
                const bool inside = have && (unsigned)(h0 + a) < (unsigned)p.H && (unsigned)(w0 + b) < (unsigned)p.W;
                const s16x4 v = __builtin_convertvector(raw[a][b], s16x4);
                d[a][b] = inside ? v : (s16x4){0, 0, 0, 0};
            }
        return;
    }
    // general path: channel counts that are not a multiple of four, the ragged last group, and
    // channel-major inputs (one byte per channel, stride H*W)
    const size_t cstride = LAYOUT == WG_NHWC ? 1 : (size_t)p.H * p.W;
#pragma unroll
    for (int a = 0; a < 6; ++a) {
        const int h = min(max(h0 + a, 0), p.H - 1);
#pragma unroll
        for (int b = 0; b < 6; ++b) {
            const int w = min(max(w0 + b, 0), p.W - 1);
            const bool inside = (unsigned)(h0 + a) < (unsigned)p.H && (unsigned)(w0 + b) < (unsigned)p.W;
            const int8_t* px = LAYOUT == WG_NHWC ? x + (((size_t)n * p.H + h) * p.W + w) * p.C
                                                 : x + (size_t)n * p.C * cstride + (size_t)h * p.W + w;
            s16x4 v = {0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c = min(c0 + i, p.C - 1);
                const short e = px[(size_t)c * cstride];
                v[i] = (inside && c0 + i < p.C) ? e : (short)0;
            }
            d[a][b] = v;
        }
    }
}

// The 1-D rule of B^T on a real 6-vector (Section 3.4, the expansion of d' = B^T d):
//   t0 = v0 - v4, t1 = v1+v2+v3+v4, t2 = -v1+v2-v3+v4, t3 = (v4-v2) + i (v3-v1), t5 = v5 - v1
// (t4 is the conjugate of t3 and never formed).
struct Line {
    s16x4 t0, t1, t2, t3r, t3i, t5;
};
__device__ inline Line bt_rule(s16x4 v0, s16x4 v1, s16x4 v2, s16x4 v3, s16x4 v4, s16x4 v5) {
    Line o;
    s16x4 s13 = v1 + v3, s24 = v2 + v4;
    o.t0 = v0 - v4;
    o.t1 = s24 + s13;
    o.t2 = s24 - s13;
    o.t3r = v4 - v2;
    o.t3i = v3 - v1;
    o.t5 = v5 - v1;
    return o;
}

// Splits values into the int8 operand planes of `MODE` and hands each plane's four
// bytes to `Sink::put(plane, bytes)`.
template <int MODE, class Sink>
struct OperandSplitter {
    Sink sink;
    __device__ inline void put(int plane, s16x4 limb) const { sink.put(plane, __builtin_convertvector(limb, s8x4)); }
    // lossless: value index q -> planes 3q (v >> 6), 3q+1 (v & 63), 3q+2 (their sum)
    __device__ inline void value(int q, s16x4 v) const {
        s16x4 hi = v >> 6, lo = v & (short)63;
        put(3 * q, hi);
        put(3 * q + 1, lo);
        put(3 * q + 2, hi + lo);
    }
    __device__ inline void limbs(int first, s16x4 v) const {
        put(first, v >> 6);
        put(first + 1, v & (short)63);
    }
    __device__ inline void real_entry(int p, s16x4 v) const {
        if (MODE == WG_LOSSLESS) value(p, v); else limbs(2 * p, v);
    }
    __device__ inline void complex_entry(int j, s16x4 re, s16x4 im) const {
        if (MODE == WG_LOSSLESS) {
            value(16 + 3 * j, re);
            value(16 + 3 * j + 1, im);
            value(16 + 3 * j + 2, re + im);   // third operand of the 3-multiplication product (Section 3.1)
        } else {
            limbs(32 + 4 * j, re);
            limbs(32 + 4 * j + 2, im);
        }
    }
};

// Transforms one tile (four channels c0..c0+3) and emits every operand plane.
template <int LAYOUT, bool VEC4, int MODE, class Sink>
__device__ inline void transform_tile(const int8_t* __restrict__ x, const Problem& p, int n, int ty, int tx, int c0,
                                      const OperandSplitter<MODE, Sink>& out) {
    s16x4 d[6][6];
    load_patch<LAYOUT, VEC4>(x, p, n, ty, tx, c0, d);
    // column pass: d'[.][b] = B^T applied down each of the six tile columns
    Line col[6];
#pragma unroll
    for (int b = 0; b < 6; ++b) col[b] = bt_rule(d[0][b], d[1][b], d[2][b], d[3][b], d[4][b], d[5][b]);
    // row pass on the real rows 0,1,2,5 of d': entries (r, {0,1,2,5}) real, (r,3) complex
#define WG_REAL_ROW(ri, field)                                                                      \
    {                                                                                               \
        Line r = bt_rule(col[0].field, col[1].field, col[2].field, col[3].field, col[4].field,      \
                         col[5].field);                                                             \
        out.real_entry(4 * ri + 0, r.t0);                                                           \
        out.real_entry(4 * ri + 1, r.t1);                                                           \
        out.real_entry(4 * ri + 2, r.t2);                                                           \
        out.real_entry(4 * ri + 3, r.t5);                                                           \
        out.complex_entry(ri, r.t3r, r.t3i);                                                        \
    }
    WG_REAL_ROW(0, t0)
    WG_REAL_ROW(1, t1)
    WG_REAL_ROW(2, t2)
    WG_REAL_ROW(3, t5)
#undef WG_REAL_ROW
    // row 3 of d' is complex, a + i b: the rule acts on a and b separately; the two
    // entries (3,3) and (3,4) mix them: (x4-x2) +- i (x3-x1).
    Line ra = bt_rule(col[0].t3r, col[1].t3r, col[2].t3r, col[3].t3r, col[4].t3r, col[5].t3r);
    Line rb = bt_rule(col[0].t3i, col[1].t3i, col[2].t3i, col[3].t3i, col[4].t3i, col[5].t3i);
    out.complex_entry(4, ra.t0, rb.t0);
    out.complex_entry(5, ra.t1, rb.t1);
    out.complex_entry(6, ra.t2, rb.t2);
    out.complex_entry(7, ra.t5, rb.t5);
    out.complex_entry(8, ra.t3r - rb.t3i, rb.t3r + ra.t3i);
    out.complex_entry(9, ra.t3r + rb.t3i, rb.t3r - ra.t3i);
}

}  // namespace wg
