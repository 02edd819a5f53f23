// Direct evaluation of the 3x3 stride-1 pad-1 convolution, the method with 144
// multiplications per 4x4 output tile and channel pair that Section 3.4 compares
// against:  y[n,k,h,w] = sum_{c,a,b} x[n,c,h+a-1,w+b-1] g[k,c,a,b].
// Serves as the on-device cross-check and the direct baseline.  Channels-last tensors with
// K % 4 == 0 and a 16-byte aligned output run on the matrix cores (operands are staged with
// 16-byte loads when C % 16 == 0 and the pointers allow it, else byte by byte); everything else
// takes the plain kernel.
#include "wg_internal.h"

namespace wg {
namespace {

// One thread per (pixel, filter), lanes along K.  Channels-last inputs whose C is a
// multiple of 4 use the packed 4 x int8 dot product.
template <int LAYOUT>
__global__ __launch_bounds__(256) void direct_conv_kernel(const int8_t* __restrict__ x,
                                                          const int8_t* __restrict__ g,
                                                          int32_t* __restrict__ y, Problem p) {
    const int k = blockIdx.y * 64 + (threadIdx.x & 63);
    const long long pix = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const long long npix = (long long)p.N * p.H * p.W;
    if (k >= p.K || pix >= npix) return;
    const int w = (int)(pix % p.W), h = (int)((pix / p.W) % p.H), n = (int)(pix / ((long long)p.W * p.H));
    int acc = 0;
    for (int a = 0; a < 3; ++a) {
        const int hh = h + a - 1;
        if (hh < 0 || hh >= p.H) continue;
        for (int b = 0; b < 3; ++b) {
            const int ww = w + b - 1;
            if (ww < 0 || ww >= p.W) continue;
            if (LAYOUT == WG_NHWC) {
                const int8_t* xp = x + (((size_t)n * p.H + hh) * p.W + ww) * p.C;
                const int8_t* gp = g + ((size_t)k * 9 + a * 3 + b) * p.C;
                int c = 0;
                if (p.C % 4 == 0)
                    for (; c < p.C; c += 4)
                        acc = __builtin_amdgcn_sdot4(*reinterpret_cast<const int*>(xp + c),
                                                     *reinterpret_cast<const int*>(gp + c), acc, false);
                for (; c < p.C; ++c) acc += (int)xp[c] * (int)gp[c];
            } else {
                const size_t plane = (size_t)p.H * p.W;
                const int8_t* xp = x + (size_t)n * p.C * plane + (size_t)hh * p.W + ww;
                const int8_t* gp = g + (size_t)k * p.C * 9 + a * 3 + b;
                for (int c = 0; c < p.C; ++c) acc += (int)xp[c * plane] * (int)gp[c * 9];
            }
        }
    }
    if (LAYOUT == WG_NHWC) y[(size_t)pix * p.K + k] = acc;
    else                   y[(((size_t)n * p.K + k) * p.H + h) * p.W + w] = acc;
}

// ---- channels-last fast path on the int8 matrix cores ---------------------------------------
// Implicit GEMM: for each of the nine taps, [64 filters x 64 channels] x [64 channels x 128
// pixels].  A workgroup owns an 8 x 16 patch of output pixels of one image and 64 filters; the
// 10 x 18 input halo and the nine filter taps of one 64-channel block are staged in LDS (rows of
// 64 bytes, the 16-byte pieces of a row XOR-swizzled by (row / 4) % 4 so that the fragment reads
// of 16 consecutive rows are conflict-free); zero padding and the ragged edges of H, W, C and K
// become zeros while staging.  Filters are the rows and pixels the columns of
// v_mfma_i32_32x32x32_i8, so that a lane ends up with four consecutive filters of one pixel: 16-byte
// stores.  Wave w multiplies patch rows 2w, 2w+1 (32 pixels) by all 64 filters.
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
constexpr int kPatchRows = 8, kPatchCols = 16, kHaloCols = kPatchCols + 2;
constexpr int kHaloPixels = (kPatchRows + 2) * kHaloCols;   // 180
constexpr int kDirectFilters = 64;

__device__ inline int row_swizzle(int row) { return (row >> 2) & 3; }

// 16 bytes of channels c..c+15 at `at` (channel 0 of a pixel or filter tap): one 16-byte load when
// the tensors allow it (VEC16), else byte by byte with channels beyond C read as zero.
template <bool VEC16>
__device__ inline v4i load_channels(const int8_t* at, int c, int C) {
    if constexpr (VEC16) {
        return *reinterpret_cast<const v4i*>(at + c);
    } else {
        v4i v = {0, 0, 0, 0};
#pragma unroll
        for (int b = 0; b < 16; ++b)
            if (c + b < C) v[b >> 2] |= (int)(uint8_t)at[c + b] << (8 * (b & 3));
        return v;
    }
}

template <bool VEC16>
__global__ __launch_bounds__(256) void direct_conv_mfma_kernel(const int8_t* __restrict__ x,
                                                               const int8_t* __restrict__ g,
                                                               int32_t* __restrict__ y, Problem p, int patches_h,
                                                               int patches_w) {
    __shared__ __attribute__((aligned(16))) int8_t halo[kHaloPixels * kCBlock];
    __shared__ __attribute__((aligned(16))) int8_t taps[9 * kDirectFilters * kCBlock];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int pw = blockIdx.x % patches_w, ph = (blockIdx.x / patches_w) % patches_h;
    const int n = blockIdx.x / (patches_w * patches_h);
    const int h0 = ph * kPatchRows, w0 = pw * kPatchCols, k0 = blockIdx.y * kDirectFilters;

    v16i acc[2];
    acc[0] = (v16i){0};
    acc[1] = (v16i){0};
    // this lane's pixel (a column of the product) and its 16-byte piece of a 32-channel step
    const int pr = 2 * wave + ((lane & 31) >> 4), pc = lane & 15, piece = lane >> 5;

    for (int cb = 0; cb < p.CB; ++cb) {
        if (cb > 0) __syncthreads();   // the previous block's fragments have been read
        constexpr v4i zero = {0, 0, 0, 0};
        v4i in[3], flt[9];
#pragma unroll
        for (int it = 0; it < 3; ++it) {
            const int item = tid + 256 * it, pix = item >> 2;
            const int h = h0 - 1 + pix / kHaloCols, w = w0 - 1 + pix % kHaloCols, c = cb * kCBlock + (item & 3) * 16;
            const bool ok = pix < kHaloPixels && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W && c < p.C;
            in[it] = zero;
            if (ok) in[it] = load_channels<VEC16>(x + (((size_t)n * p.H + h) * p.W + w) * p.C, c, p.C);
        }
#pragma unroll
        for (int it = 0; it < 9; ++it) {
            const int item = tid + 256 * it, kt = item >> 2;   // kt = filter * 9 + tap: contiguous in memory
            const int kk = k0 + kt / 9, c = cb * kCBlock + (item & 3) * 16;
            flt[it] = zero;
            if (kk < p.K && c < p.C) flt[it] = load_channels<VEC16>(g + ((size_t)k0 * 9 + kt) * p.C, c, p.C);
        }
#pragma unroll
        for (int it = 0; it < 3; ++it) {
            const int item = tid + 256 * it, pix = item >> 2;
            if (pix < kHaloPixels)
                *reinterpret_cast<v4i*>(halo + pix * kCBlock + (((item & 3) ^ row_swizzle(pix)) * 16)) = in[it];
        }
#pragma unroll
        for (int it = 0; it < 9; ++it) {
            const int item = tid + 256 * it, kt = item >> 2;
            const int row = (kt % 9) * kDirectFilters + kt / 9;   // [tap][filter]
            *reinterpret_cast<v4i*>(taps + row * kCBlock + (((item & 3) ^ row_swizzle(row)) * 16)) = flt[it];
        }
        __syncthreads();
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
            const int hp = (pr + tap / 3) * kHaloCols + pc + tap % 3;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const int at = 2 * ks + piece;
                const v4i b = *reinterpret_cast<const v4i*>(halo + hp * kCBlock + ((at ^ row_swizzle(hp)) * 16));
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    const int row = tap * kDirectFilters + mt * 32 + (lane & 31);
                    const v4i a = *reinterpret_cast<const v4i*>(taps + row * kCBlock + ((at ^ row_swizzle(row)) * 16));
                    acc[mt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[mt], 0, 0, 0);
                }
            }
        }
    }
    // register i of a 32x32 product: row (filter) 8 (i / 4) + 4 (lane / 32) + i % 4, column (pixel) lane % 32
    const int h = h0 + pr, w = w0 + pc;
    if (h >= p.H || w >= p.W) return;
    int32_t* out = y + (((size_t)n * p.H + h) * p.W + w) * p.K;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int kk = k0 + mt * 32 + 8 * q + 4 * piece;
            if (kk < p.K)
                *reinterpret_cast<v4i*>(out + kk) = (v4i){acc[mt][4 * q], acc[mt][4 * q + 1], acc[mt][4 * q + 2], acc[mt][4 * q + 3]};
        }
}

// v = (y + 2^(shift-1)) >> shift, clamp, optional 2x2 max-pool; one thread per output element.
template <int LAYOUT>
__global__ __launch_bounds__(256) void requant_relu_pool_kernel(const int32_t* __restrict__ y,
                                                                int8_t* __restrict__ out, int N, int K,
                                                                int H, int W, int shift, int lo, int pool) {
    const int Ho = pool ? H / 2 : H, Wo = pool ? W / 2 : W;
    const size_t total = (size_t)N * K * Ho * Wo;
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    int n, k, h, w;
    if (LAYOUT == WG_NHWC) {
        k = (int)(i % K); w = (int)((i / K) % Wo); h = (int)((i / ((size_t)K * Wo)) % Ho);
        n = (int)(i / ((size_t)K * Wo * Ho));
    } else {
        w = (int)(i % Wo); h = (int)((i / Wo) % Ho); k = (int)((i / ((size_t)Wo * Ho)) % K);
        n = (int)(i / ((size_t)Wo * Ho * K));
    }
    const int span = pool ? 2 : 1;
    const int rnd = shift > 0 ? (1 << (shift - 1)) : 0;
    int best = -129;
    for (int a = 0; a < span; ++a)
        for (int b = 0; b < span; ++b) {
            const int hh = pool ? 2 * h + a : h, ww = pool ? 2 * w + b : w;
            const int32_t v0 = LAYOUT == WG_NHWC ? y[(((size_t)n * H + hh) * W + ww) * K + k]
                                                 : y[(((size_t)n * K + k) * H + hh) * W + ww];
            int v = (int)(((long long)v0 + rnd) >> shift);
            v = v < lo ? lo : (v > 127 ? 127 : v);
            best = v > best ? v : best;
        }
    out[i] = (int8_t)best;
}

}  // namespace

hipError_t launch_direct_conv(const int8_t* x, const int8_t* w, int32_t* y, const Problem& p, int layout,
                              hipStream_t s) {
    auto aligned16 = [](const void* q) { return reinterpret_cast<uintptr_t>(q) % 16 == 0; };
    if (layout == WG_NHWC && p.K % 4 == 0 && aligned16(y)) {
        const int patches_h = ceil_div(p.H, kPatchRows), patches_w = ceil_div(p.W, kPatchCols);
        dim3 grid((unsigned)(p.N * patches_h * patches_w), ceil_div(p.K, kDirectFilters));
        if (p.C % 16 == 0 && aligned16(x) && aligned16(w))
            direct_conv_mfma_kernel<true><<<grid, 256, 0, s>>>(x, w, y, p, patches_h, patches_w);
        else
            direct_conv_mfma_kernel<false><<<grid, 256, 0, s>>>(x, w, y, p, patches_h, patches_w);
        return hipGetLastError();
    }
    const long long npix = (long long)p.N * p.H * p.W;
    dim3 grid((unsigned)((npix + 3) / 4), ceil_div(p.K, 64));
    if (layout == WG_NHWC) direct_conv_kernel<WG_NHWC><<<grid, 256, 0, s>>>(x, w, y, p);
    else                   direct_conv_kernel<WG_NCHW><<<grid, 256, 0, s>>>(x, w, y, p);
    return hipGetLastError();
}

hipError_t launch_requant_relu_pool(const int32_t* y, int8_t* out, int N, int K, int H, int W, int layout,
                                    int shift, int relu, int pool, hipStream_t s) {
    const size_t total = (size_t)N * K * (pool ? H / 2 : H) * (pool ? W / 2 : W);
    const unsigned blocks = (unsigned)((total + 255) / 256);
    const int lo = relu ? 0 : -128;
    if (layout == WG_NHWC) requant_relu_pool_kernel<WG_NHWC><<<blocks, 256, 0, s>>>(y, out, N, K, H, W, shift, lo, pool);
    else                   requant_relu_pool_kernel<WG_NCHW><<<blocks, 256, 0, s>>>(y, out, N, K, H, W, shift, lo, pool);
    return hipGetLastError();
}

}  // namespace wg
