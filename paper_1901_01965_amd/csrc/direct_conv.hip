// Direct evaluation of the 3x3 stride-1 pad-1 convolution, the method with 144
// multiplications per 4x4 output tile and channel pair that Section 3.4 compares
// against:  y[n,k,h,w] = sum_{c,a,b} x[n,c,h+a-1,w+b-1] g[k,c,a,b].
// Serves as the on-device cross-check and the direct baseline.
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
