// Small device-side pieces shared by the single-kernel convolution variants.
#pragma once
#include <type_traits>
#include <utility>

#include "input_transform_core.h"

namespace wg {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kTileBlock = 16;                      // tiles per workgroup (one side of the 16x16x64 matrix-core product)
constexpr int kPlaneBytes = kTileBlock * kCBlock;   // one operand plane of a tile block in LDS

// LDS operand plane: the 16-byte piece holding 16 consecutive channels (group c16) of a tile
// sits in slot c16*16 + ((tile + 4*c16) & 15); lane l of a wave reads slot(l/16, l%16), which
// tiles the plane without bank conflicts for the 4-byte writes as well as the 16-byte reads.
__device__ inline int lds_slot(int c16, int tile) { return c16 * 16 + ((tile + 4 * c16) & 15); }

struct LdsPlaneSink {
    int8_t* base;
    __device__ inline void put(int plane, uint32_t bytes) const {
        *reinterpret_cast<uint32_t*>(base + plane * kPlaneBytes) = bytes;
    }
};

// compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(<N-1>)
template <class F, int... Is>
__device__ inline void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ inline void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// The optional int8 epilogue: v = (y + round) >> shift clamped to [lo, 127].
__device__ inline int requantise(int y, const Int8Epilogue& q) {
    return min(max((y + q.round) >> q.shift, q.lo), 127);
}
__device__ inline v4i requantise(v4i y, const Int8Epilogue& q) {
    y = (y + q.round) >> q.shift;
    const v4i lo = {q.lo, q.lo, q.lo, q.lo}, hi = {127, 127, 127, 127};
    return __builtin_elementwise_min(__builtin_elementwise_max(y, lo), hi);
}
__device__ inline uint32_t pack_bytes(v4i v) {
    return (uint32_t)(v[0] & 0xff) | ((uint32_t)(v[1] & 0xff) << 8) | ((uint32_t)(v[2] & 0xff) << 16) | ((uint32_t)v[3] << 24);
}

// Patch loads of the role-specialised kernels go through a buffer descriptor over the activation
// tensor: a load whose offset lies beyond the tensor returns zero, so a pixel outside the image
// (pad 1, ragged tiles) is an offset that can never be in range instead of a select per pixel and
// channel block.  Offsets of rows and columns outside the image are kOutsideOffset; they are
// combined with a saturating addition, so that any sum with an outside part stays at or above
// 2^31, more than the tensor can hold (the host checks N*C*H*W < 2^31).
constexpr uint32_t kOutsideOffset = 0x80000000u;
constexpr int kRawBufferWord3 = 0x00020000;   // untyped 32-bit data, as for every raw buffer on this target
__device__ inline __amdgpu_buffer_rsrc_t activation_buffer(const int8_t* x, const Problem& p) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(x), 0, p.N * p.H * p.W * p.C, kRawBufferWord3);
}

// Offsets (relative to x, channel c_lane of the pixel) of the 6x6 patch of tile (n, ty, tx).
__device__ inline void patch_offsets(const Problem& p, int n, int ty, int tx, int c_lane, uint32_t pixel[36]) {
    const int h0 = 4 * ty - 1, w0 = 4 * tx - 1;
    const uint32_t image = (uint32_t)n * (uint32_t)p.H * (uint32_t)p.W * (uint32_t)p.C + (uint32_t)c_lane;
    uint32_t row_off[6], col_off[6];
#pragma unroll
    for (int a = 0; a < 6; ++a) {
        row_off[a] = (unsigned)(h0 + a) < (unsigned)p.H ? image + (uint32_t)(h0 + a) * (uint32_t)p.W * (uint32_t)p.C : kOutsideOffset;
        col_off[a] = (unsigned)(w0 + a) < (unsigned)p.W ? (uint32_t)(w0 + a) * (uint32_t)p.C : kOutsideOffset;
    }
#pragma unroll
    for (int a = 0; a < 6; ++a)
#pragma unroll
        for (int b = 0; b < 6; ++b) pixel[6 * a + b] = __builtin_elementwise_add_sat(row_off[a], col_off[b]);
}
// One channel block of the patch: 36 loads, nothing waits for them here.  pixel[] holds the
// offsets of the lane's channel group in channel block 0; the block is a uniform offset on top.
// Only the last channel block of a C that is not a multiple of 64 has channel groups beyond C:
// there (a uniform branch) such a lane asks for the outside offset, so that it gets zeros and
// never touches memory next to the tensor.
__device__ inline void request_patch(__amdgpu_buffer_rsrc_t xbuf, const Problem& p, const uint32_t pixel[36], int cb,
                                     int c_lane, uint32_t patch[6][6]) {
    if ((cb + 1) * kCBlock > p.C) {
        const bool have = cb * kCBlock + c_lane < p.C;
#pragma unroll
        for (int i = 0; i < 36; ++i)
            patch[i / 6][i % 6] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(xbuf, have ? pixel[i] : kOutsideOffset, cb * kCBlock, 0);
    } else {
#pragma unroll
        for (int i = 0; i < 36; ++i)
            patch[i / 6][i % 6] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(xbuf, pixel[i], cb * kCBlock, 0);
    }
}
// u = x + 128 on every byte; what does not exist arrived as zeros, i.e. x = 0.
__device__ inline void bias_buffer_patch(uint32_t patch[6][6]) {
#pragma unroll
    for (int i = 0; i < 36; ++i) patch[i / 6][i % 6] ^= kBiasBytes;
}

// Row rule of A^T on (m0, m1, m2, m3, conj(m3), m5) with m0,m1,m2,m5 real:
//   z0 = m0+m1+m2+2Re m3, z1 = m1-m2-2Im m3, z2 = m1+m2-2Re m3, z3 = m1-m2+2Im m3+m5
template <class V>
__device__ inline void at_rule(V m0, V m1, V m2, V m3r, V m3i, V m5, V z[4]) {
    const V s = m1 + m2, d = m1 - m2;
    z[0] = m0 + s + 2 * m3r;
    z[1] = d - 2 * m3i;
    z[2] = s - 2 * m3r;
    z[3] = d + 2 * m3i + m5;
}

// A finished row of M is reduced by the row rule and enters the 16 outputs with the
// column-rule coefficients of A^T.  Real rows 0,1,2,5 (ROW = 0..3; entries m0,m1,m2,m5 real
// at positions 0..3, complex m3 at position 4): row 0 -> y0; rows 1, 2 -> (+,+,+,+), (+,-,+,-);
// row 5 -> y3.  The complex row 3 (ROW = 4; e0,e1,e2,e5 at positions 0..3, e3 = M[3][3] and
// e4 = M[3][4] at 4, 5; row 4 of M is its conjugate): y0 += 2Re z, y1 -= 2Im z, y2 -= 2Re z,
// y3 += 2Im z.
template <int ROW, class V>
__device__ inline void finish_row(const V (&er)[6], const V (&ei)[6], V (&Y)[16]) {
    if constexpr (ROW < 4) {
        V z[4];
        at_rule(er[0], er[1], er[2], er[4], ei[4], er[3], z);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (ROW == 0) Y[j] += z[j];
            if (ROW == 1) { Y[j] += z[j]; Y[4 + j] += z[j]; Y[8 + j] += z[j]; Y[12 + j] += z[j]; }
            if (ROW == 2) { Y[j] += z[j]; Y[4 + j] -= z[j]; Y[8 + j] += z[j]; Y[12 + j] -= z[j]; }
            if (ROW == 3) Y[12 + j] += z[j];
        }
    } else {
        const V sr = er[4] + er[5], si = ei[4] + ei[5], dr = er[4] - er[5], di = ei[4] - ei[5];
        const V ar = er[1] + er[2], ai = ei[1] + ei[2], br = er[1] - er[2], bi = ei[1] - ei[2];
        V zr[4], zi[4];
        zr[0] = er[0] + ar + sr;   zi[0] = ei[0] + ai + si;
        zr[1] = br - di;           zi[1] = bi + dr;            // (e1-e2) + i (e3-e4)
        zr[2] = ar - sr;           zi[2] = ai - si;
        zr[3] = br + di + er[3];   zi[3] = bi - dr + ei[3];    // (e1-e2) - i (e3-e4) + e5
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            Y[j] += 2 * zr[j];
            Y[4 + j] -= 2 * zi[j];
            Y[8 + j] -= 2 * zr[j];
            Y[12 + j] += 2 * zi[j];
        }
    }
}

}  // namespace wg
