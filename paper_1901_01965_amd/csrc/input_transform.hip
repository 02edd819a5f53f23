// Input transform D = B^T d B of the overlapping 6x6 tiles (Section 3.3), using
// the row expansion and conjugate structure of Section 3.4: only the 26 free
// entries are formed, with additions and subtractions alone, four channels at a
// time in packed 16-bit lanes; each 12-bit result is split into the int8 operand
// planes the contraction consumes.
#include "wg_internal.h"

namespace wg {
namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef signed char s8x4 __attribute__((ext_vector_type(4)));

// Four consecutive channels of one pixel, zero outside the image or beyond C.
template <int LAYOUT>
__device__ inline s16x4 load_px(const int8_t* x, const Problem& p, int n, int h, int w, int c0, bool vec_ok) {
    s16x4 r = {0, 0, 0, 0};
    if (h < 0 || h >= p.H || w < 0 || w >= p.W) return r;
    if (LAYOUT == WG_NHWC) {
        const int8_t* px = x + (((size_t)n * p.H + h) * p.W + w) * p.C + c0;
        if (vec_ok) {
            s8x4 v = *reinterpret_cast<const s8x4*>(px);
            return __builtin_convertvector(v, s16x4);
        }
        for (int i = 0; i < 4; ++i)
            if (c0 + i < p.C) r[i] = px[i];
    } else {
        const size_t plane = (size_t)p.H * p.W;
        const int8_t* px = x + ((size_t)n * p.C + c0) * plane + (size_t)h * p.W + w;
        for (int i = 0; i < 4; ++i)
            if (c0 + i < p.C) r[i] = px[i * plane];
    }
    return r;
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

template <int MODE>
struct PlaneWriter {
    int8_t* base;          // V + ((cb * Tp + t) * 64 + 4 * cq)
    size_t plane_stride;   // CB * Tp * 64
    __device__ inline void put(int plane, s16x4 limb) const {
        *reinterpret_cast<s8x4*>(base + (size_t)plane * plane_stride) = __builtin_convertvector(limb, s8x4);
    }
    // lossless: value index q -> planes 3q (high), 3q+1 (low), 3q+2 (high+low)
    __device__ inline void value(int q, s16x4 v) const {
        s16x4 hi = v >> 6, lo = v & (short)63;
        put(3 * q, hi);
        put(3 * q + 1, lo);
        put(3 * q + 2, hi + lo);
    }
    // scaled: two limbs at planes `first`, `first + 1`
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
            value(16 + 3 * j + 2, re + im);   // third operand of the 3-multiplication product
        } else {
            limbs(32 + 4 * j, re);
            limbs(32 + 4 * j + 2, im);
        }
    }
};

// One thread per (tile, group of four channels); a 256-thread block covers 16 tiles
// of one 64-channel block, so each wave stores 256 contiguous bytes per operand plane.
template <int LAYOUT, int MODE>
__global__ __launch_bounds__(256) void input_transform_kernel(const int8_t* __restrict__ x,
                                                              int8_t* __restrict__ V, Problem p) {
    const int cq = threadIdx.x & 15;
    const int t = blockIdx.x * 16 + (threadIdx.x >> 4);
    const int cb = blockIdx.y;
    if (t >= p.T) return;
    const int tx = t % p.TW, ty = (t / p.TW) % p.TH, n = t / (p.TW * p.TH);
    const int c0 = cb * kCBlock + 4 * cq;
    const bool vec_ok = (p.C % 4 == 0) && (c0 + 3 < p.C);

    // column pass: d'[.][b] = B^T applied down each of the six tile columns
    Line col[6];
#pragma unroll
    for (int b = 0; b < 6; ++b) {
        s16x4 v[6];
#pragma unroll
        for (int a = 0; a < 6; ++a) v[a] = load_px<LAYOUT>(x, p, n, 4 * ty - 1 + a, 4 * tx - 1 + b, c0, vec_ok);
        col[b] = bt_rule(v[0], v[1], v[2], v[3], v[4], v[5]);
    }

    PlaneWriter<MODE> out;
    out.base = V + (((size_t)cb * p.Tp + t) * kCBlock + 4 * cq);
    out.plane_stride = (size_t)p.CB * p.Tp * kCBlock;

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

__global__ void unpack_activation_planes_kernel(const int8_t* V, int8_t* dense, Problem p, int nplanes) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)nplanes * p.T * p.C;
    if (i >= total) return;
    int c = (int)(i % p.C);
    int t = (int)((i / p.C) % p.T);
    int pl = (int)(i / ((size_t)p.C * p.T));
    dense[i] = V[(((size_t)pl * p.CB + (c >> 6)) * p.Tp + t) * kCBlock + (c & 63)];
}

}  // namespace

hipError_t launch_input_transform(const int8_t* x, const Problem& p, int layout, int mode, int8_t* V,
                                  hipStream_t s) {
    dim3 grid(ceil_div(p.T, 16), p.CB);
    if (layout == WG_NHWC) {
        if (mode == WG_LOSSLESS) input_transform_kernel<WG_NHWC, WG_LOSSLESS><<<grid, 256, 0, s>>>(x, V, p);
        else                     input_transform_kernel<WG_NHWC, WG_SCALED><<<grid, 256, 0, s>>>(x, V, p);
    } else {
        if (mode == WG_LOSSLESS) input_transform_kernel<WG_NCHW, WG_LOSSLESS><<<grid, 256, 0, s>>>(x, V, p);
        else                     input_transform_kernel<WG_NCHW, WG_SCALED><<<grid, 256, 0, s>>>(x, V, p);
    }
    return hipGetLastError();
}

hipError_t launch_unpack_activation_planes(const int8_t* V, int8_t* dense, const Problem& p, int mode,
                                           hipStream_t s) {
    const int nplanes = num_activation_planes(mode);
    size_t total = (size_t)nplanes * p.T * p.C;
    unpack_activation_planes_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(V, dense, p, nplanes);
    return hipGetLastError();
}

}  // namespace wg
