// The arithmetic of the input transform D = B^T d B (Section 3.3) on the 26 free
// entries (Section 3.4), shared by the stand-alone transform kernel and the
// fused convolution kernel.  Four channels are processed at a time in packed
// 16-bit lanes; `Sink` decides where each int8 operand plane goes.
//
// Activations are handled in the biased form u = x + 128 (one XOR on the packed
// bytes, so that unpacking is a plain zero extension).  A constant patch maps to
// zero at every entry of B^T d B except (1,1), where the sixteen +1 coefficients
// add up: D(u) = D(x) + 2048 at (1,1) only, so the bias is removed by one
// subtraction.  Padding pixels and channels beyond C carry the bias value 128.
// uint8 tensors with a zero point z (Section 4.1) are the same form with bias z and no XOR.
#pragma once
#include "wg_internal.h"

namespace wg {

typedef short s16x2 __attribute__((ext_vector_type(2)));

// four channels: a = (c0, c1), b = (c2, c3)
struct Quad {
    s16x2 a, b;
};
__device__ inline Quad operator+(Quad x, Quad y) { return Quad{x.a + y.a, x.b + y.b}; }
__device__ inline Quad operator-(Quad x, Quad y) { return Quad{x.a - y.a, x.b - y.b}; }

__device__ inline uint32_t as_u32(s16x2 v) { return __builtin_bit_cast(uint32_t, v); }
__device__ inline s16x2 as_s16x2(uint32_t v) { return __builtin_bit_cast(s16x2, v); }

// bytes (u0,u1,u2,u3) -> 16-bit lanes (u0,u1), (u2,u3), zero extended
__device__ inline Quad unpack_u8x4(uint32_t u) {
    return Quad{as_s16x2(__builtin_amdgcn_perm(0u, u, 0x0c010c00u)), as_s16x2(__builtin_amdgcn_perm(0u, u, 0x0c030c02u))};
}
// low bytes of the four 16-bit lanes -> one dword (c0,c1,c2,c3)
__device__ inline uint32_t pack_low_bytes(Quad v) { return __builtin_amdgcn_perm(as_u32(v.b), as_u32(v.a), 0x06040200u); }
// their high bytes
__device__ inline uint32_t pack_high_bytes(Quad v) { return __builtin_amdgcn_perm(as_u32(v.b), as_u32(v.a), 0x07050301u); }

constexpr uint32_t kBiasBytes = 0x80808080u;

// How the stored bytes encode the integers x that are convolved.  The transform always works on
// non-negative bytes u = x + bias; the encoding says how a stored byte becomes u (an XOR), which
// byte stands for x = 0 (what padding pixels and channels beyond C must read as), and what the
// bias leaves at entry (1,1), in both 16-bit lanes.
//   SignedInt8:   x is the byte read as int8, u = byte ^ 0x80 = x + 128;
//   ZeroPointU8:  the quantised tensors of Section 4.1: x = byte - zero_point, an integer in
//                 [-255, 255]; u is the byte itself, the bias is the zero point.
struct SignedInt8 {
    static constexpr uint32_t kMagic = kBlobMagic;       // goes with blobs of signed int8 filters
    __device__ inline uint32_t flip() const { return kBiasBytes; }
    __device__ inline uint32_t absent_stored() const { return 0u; }     // the stored byte of x = 0 ...
    __device__ inline uint32_t absent() const { return kBiasBytes; }    // ... and its u, in all four bytes
    __device__ inline uint32_t bias11() const { return 0x08000800u; }   // 16 * 128
};
struct ZeroPointU8 {
    static constexpr uint32_t kMagic = kBlobMagicInt9;   // goes with blobs of uint8 filters with a zero point
    uint32_t zero_bytes;     // the zero point in all four bytes
    uint32_t zero_sixteen;   // 16 * zero point in both 16-bit halves
    __device__ inline uint32_t flip() const { return 0u; }
    __device__ inline uint32_t absent_stored() const { return zero_bytes; }
    __device__ inline uint32_t absent() const { return zero_bytes; }
    __device__ inline uint32_t bias11() const { return zero_sixteen; }
};
inline ZeroPointU8 make_zero_point(int z) { return ZeroPointU8{(uint32_t)z * 0x01010101u, (uint32_t)(16 * z) * 0x00010001u}; }

// The 6x6 input patch of one tile, four consecutive channels c0..c0+3 per pixel, as raw loads:
// addresses are clamped into the image so no load sits behind a branch and nothing here waits
// for data; bias_patch() then applies the bias and replaces out-of-range pixels.
// VEC4 (channels-last input whose C is a multiple of four, chosen on the host): one 4-byte
// load per pixel; a channel group is then either wholly inside or wholly beyond C.
template <int LAYOUT, bool VEC4, class ENC = SignedInt8>
__device__ inline void load_patch(const int8_t* __restrict__ x, const Problem& p, int n, int ty, int tx, int c0,
                                  uint32_t u[6][6], const ENC enc = ENC{}) {
    // Offsets fit 32 bits (the host checks N*C*H*W < 2^31): one multiply per patch row and
    // column instead of 64-bit address arithmetic per pixel.
    const int h0 = 4 * ty - 1, w0 = 4 * tx - 1;
    const uint32_t pixel_stride = LAYOUT == WG_NHWC ? (uint32_t)p.C : 1u;
    uint32_t row_off[6], col_off[6];
#pragma unroll
    for (int a = 0; a < 6; ++a) {
        row_off[a] = (uint32_t)min(max(h0 + a, 0), p.H - 1) * (uint32_t)p.W * pixel_stride;
        col_off[a] = (uint32_t)min(max(w0 + a, 0), p.W - 1) * pixel_stride;
    }
    if constexpr (VEC4) {
        static_assert(LAYOUT == WG_NHWC, "4-byte pixel loads need channels-last input");
        const int8_t* img = x + (size_t)n * p.H * p.W * p.C + (c0 < p.C ? c0 : 0);
#pragma unroll
        for (int a = 0; a < 6; ++a)
#pragma unroll
            for (int b = 0; b < 6; ++b) u[a][b] = *reinterpret_cast<const uint32_t*>(img + (row_off[a] + col_off[b]));
    } else {
        // general path: channel counts that are not a multiple of four, and channel-major inputs
        // (one byte per channel, stride H*W)
        const uint32_t cstride = LAYOUT == WG_NHWC ? 1u : (uint32_t)p.H * (uint32_t)p.W;
        const int8_t* img = x + (size_t)n * p.C * p.H * p.W;
        uint32_t chan_off[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) chan_off[i] = (uint32_t)min(c0 + i, p.C - 1) * cstride;
#pragma unroll
        for (int a = 0; a < 6; ++a)
#pragma unroll
            for (int b = 0; b < 6; ++b) {
                uint32_t word = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t e = (uint8_t)img[row_off[a] + col_off[b] + chan_off[i]];
                    word |= (c0 + i < p.C ? e : (enc.absent_stored() & 0xffu)) << (8 * i);   // x = 0 beyond C
                }
                u[a][b] = word;
            }
    }
}

// u = x + bias on every byte; pixels outside the image (pad 1) and channel groups beyond C
// become the bias value itself, i.e. x = 0.
template <class ENC = SignedInt8>
__device__ inline void bias_patch(const Problem& p, int ty, int tx, int c0, uint32_t u[6][6], const ENC enc = ENC{}) {
    const int h0 = 4 * ty - 1, w0 = 4 * tx - 1;
    const bool have = c0 < p.C;
#pragma unroll
    for (int a = 0; a < 6; ++a)
#pragma unroll
        for (int b = 0; b < 6; ++b) {
            const bool inside = have && (unsigned)(h0 + a) < (unsigned)p.H && (unsigned)(w0 + b) < (unsigned)p.W;
            u[a][b] = inside ? (u[a][b] ^ enc.flip()) : enc.absent();
        }
}

// The 1-D rule of B^T on a real 6-vector (Section 3.4, the expansion of d' = B^T d):
//   t0 = v0 - v4, t1 = v1+v2+v3+v4, t2 = -v1+v2-v3+v4, t3 = (v4-v2) + i (v3-v1), t5 = v5 - v1
// (t4 is the conjugate of t3 and never formed).
struct Line {
    Quad t0, t1, t2, t3r, t3i, t5;
};
__device__ inline Line bt_rule(Quad v0, Quad v1, Quad v2, Quad v3, Quad v4, Quad v5) {
    Line o;
    const Quad s13 = v1 + v3, s24 = v2 + v4;
    o.t0 = v0 - v4;
    o.t1 = s24 + s13;
    o.t2 = s24 - s13;
    o.t3r = v4 - v2;
    o.t3i = v3 - v1;
    o.t5 = v5 - v1;
    return o;
}

// How a 12-bit value v = 64 h + l is handed to the matrix cores:
//   kSplitKaratsuba: three planes per value, h, l and h + l (the middle operand of the
//                    three-multiplication split of Section 3.1), and a third value Re+Im per
//                    complex entry (the extra operand of the three-multiplication complex
//                    product): 138 planes, the lossless staged layout;
//   kSplitTwoLimb:   two planes per value, h and l: real entry p -> 2p, 2p+1; complex entry j
//                    -> 32+4j + {Re h, Re l, Im h, Im l}: 72 planes;
//   kSplitByteLimbs: the same 72 planes with v = 256 h + l, l the low byte of v read as a signed
//                    int8 and h = (v + 128) >> 8 in [-8, 8]: both limbs are bytes of a register
//                    already, so the split costs one addition instead of a shift and a mask.  Used
//                    where the other operand is a single int8 (scaled mode inside one kernel): the
//                    two limb products then simply carry the weights 256 and 1.
constexpr int kSplitKaratsuba = 0, kSplitTwoLimb = 1, kSplitByteLimbs = 2;
constexpr int kByteLimbShift = 8;

template <int SPLIT, class Sink>
struct OperandSplitter {
    Sink sink;
    __device__ inline static Quad high(Quad v) { return Quad{v.a >> 6, v.b >> 6}; }
    __device__ inline static Quad low(Quad v) {
        return Quad{as_s16x2(as_u32(v.a) & 0x003f003fu), as_s16x2(as_u32(v.b) & 0x003f003fu)};
    }
    __device__ inline void value(int q, Quad v) const {   // planes 3q, 3q+1, 3q+2
        const Quad hi = high(v), lo = low(v);
        sink.put(3 * q, pack_low_bytes(hi));
        sink.put(3 * q + 1, pack_low_bytes(lo));
        sink.put(3 * q + 2, pack_low_bytes(hi + lo));
    }
    __device__ inline void limbs(int first, Quad v) const {
        if (SPLIT == kSplitByteLimbs) {
            const s16x2 half = {128, 128};
            sink.put(first, pack_high_bytes(Quad{v.a + half, v.b + half}));
            sink.put(first + 1, pack_low_bytes(v));
        } else {
            sink.put(first, pack_low_bytes(high(v)));
            sink.put(first + 1, pack_low_bytes(v) & 0x3f3f3f3fu);   // v & 63 on all four channels at once
        }
    }
    __device__ inline void real_entry(int p, Quad v) const {
        if (SPLIT == kSplitKaratsuba) value(p, v); else limbs(2 * p, v);
    }
    __device__ inline void complex_entry(int j, Quad re, Quad im) const {
        if (SPLIT == kSplitKaratsuba) {
            value(16 + 3 * j, re);
            value(16 + 3 * j + 1, im);
            value(16 + 3 * j + 2, re + im);
        } else {
            limbs(32 + 4 * j, re);
            limbs(32 + 4 * j + 2, im);
        }
    }
};

// Transforms one loaded patch (four channels) and hands every free entry to `out`
// (real_entry(p, v), complex_entry(j, re, im)): an OperandSplitter emits the operand planes.
template <class Out, class ENC = SignedInt8>
__device__ inline void transform_patch(const uint32_t u[6][6], const Out& out, const ENC enc = ENC{}) {
    // column pass: d'[.][b] = B^T applied down each of the six tile columns
    Line col[6];
#pragma unroll
    for (int b = 0; b < 6; ++b)
        col[b] = bt_rule(unpack_u8x4(u[0][b]), unpack_u8x4(u[1][b]), unpack_u8x4(u[2][b]), unpack_u8x4(u[3][b]),
                         unpack_u8x4(u[4][b]), unpack_u8x4(u[5][b]));
    const s16x2 bias11 = as_s16x2(enc.bias11());   // what the bias leaves at entry (1,1): 16 * 128 for signed int8
    // row pass on the real rows 0,1,2,5 of d': entries (r, {0,1,2,5}) real, (r,3) complex
#define WG_REAL_ROW(ri, field)                                                                      \
    {                                                                                               \
        Line r = bt_rule(col[0].field, col[1].field, col[2].field, col[3].field, col[4].field,      \
                         col[5].field);                                                             \
        if (ri == 1) r.t1 = Quad{r.t1.a - bias11, r.t1.b - bias11};                                 \
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
    const Line ra = bt_rule(col[0].t3r, col[1].t3r, col[2].t3r, col[3].t3r, col[4].t3r, col[5].t3r);
    const Line rb = bt_rule(col[0].t3i, col[1].t3i, col[2].t3i, col[3].t3i, col[4].t3i, col[5].t3i);
    out.complex_entry(4, ra.t0, rb.t0);
    out.complex_entry(5, ra.t1, rb.t1);
    out.complex_entry(6, ra.t2, rb.t2);
    out.complex_entry(7, ra.t5, rb.t5);
    out.complex_entry(8, ra.t3r - rb.t3i, rb.t3r + ra.t3i);
    out.complex_entry(9, ra.t3r + rb.t3i, rb.t3r - ra.t3i);
}

}  // namespace wg

namespace wg {
// Loads and transforms one tile (four channels c0..c0+3).
template <int LAYOUT, bool VEC4, int SPLIT, class Sink>
__device__ inline void transform_tile(const int8_t* __restrict__ x, const Problem& p, int n, int ty, int tx, int c0,
                                      const OperandSplitter<SPLIT, Sink>& out) {
    uint32_t u[6][6];
    load_patch<LAYOUT, VEC4>(x, p, n, ty, tx, c0, u);
    bias_patch(p, ty, tx, c0, u);
    transform_patch(u, out);
}
}  // namespace wg
