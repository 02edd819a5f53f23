// Input transform D = B^T d B of the overlapping 6x6 tiles (Section 3.3), using
// the row expansion and conjugate structure of Section 3.4: only the 26 free
// entries are formed, with additions and subtractions alone, four channels at a
// time in packed 16-bit lanes; each 12-bit result is split into the int8 operand
// planes the contraction consumes.
#include "input_transform_core.h"

namespace wg {
namespace {

// Writes one operand plane's four bytes into the workspace array V [planes][CB][Tp][64].
struct GlobalPlaneSink {
    int8_t* base;          // V + ((cb * Tp + t) * 64 + 4 * cq)
    size_t plane_stride;   // CB * Tp * 64
    __device__ inline void put(int plane, uint32_t bytes) const {
        *reinterpret_cast<uint32_t*>(base + (size_t)plane * plane_stride) = bytes;
    }
};

// One thread per (tile, group of four channels); a 256-thread block covers 16 tiles
// of one 64-channel block, so each wave stores 256 contiguous bytes per operand plane.
template <int LAYOUT, bool VEC4, int MODE>
__global__ __launch_bounds__(256) void input_transform_kernel(const int8_t* __restrict__ x,
                                                              int8_t* __restrict__ V, Problem p) {
    const int cq = threadIdx.x & 15;
    const int t = blockIdx.x * 16 + (threadIdx.x >> 4);
    const int cb = blockIdx.y;
    if (t >= p.T) return;
    int n, ty, tx;
    decode_tile(p, t, n, ty, tx);
    constexpr int SPLIT = MODE == WG_LOSSLESS ? kSplitKaratsuba : kSplitTwoLimb;
    OperandSplitter<SPLIT, GlobalPlaneSink> out;
    out.sink.base = V + (((size_t)cb * p.Tp + t) * kCBlock + 4 * cq);
    out.sink.plane_stride = (size_t)p.CB * p.Tp * kCBlock;
    transform_tile<LAYOUT, VEC4, SPLIT>(x, p, n, ty, tx, cb * kCBlock + 4 * cq, out);
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
    if (layout == WG_NHWC && p.C % 4 == 0) {
        if (mode == WG_LOSSLESS) input_transform_kernel<WG_NHWC, true, WG_LOSSLESS><<<grid, 256, 0, s>>>(x, V, p);
        else                     input_transform_kernel<WG_NHWC, true, WG_SCALED><<<grid, 256, 0, s>>>(x, V, p);
    } else if (layout == WG_NHWC) {
        if (mode == WG_LOSSLESS) input_transform_kernel<WG_NHWC, false, WG_LOSSLESS><<<grid, 256, 0, s>>>(x, V, p);
        else                     input_transform_kernel<WG_NHWC, false, WG_SCALED><<<grid, 256, 0, s>>>(x, V, p);
    } else {
        if (mode == WG_LOSSLESS) input_transform_kernel<WG_NCHW, false, WG_LOSSLESS><<<grid, 256, 0, s>>>(x, V, p);
        else                     input_transform_kernel<WG_NCHW, false, WG_SCALED><<<grid, 256, 0, s>>>(x, V, p);
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
