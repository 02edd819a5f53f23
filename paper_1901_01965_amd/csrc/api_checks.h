// Argument checks shared by the translation units that implement the C ABI: everything is decided on
// the host before the first launch.
#pragma once
#include "wg_internal.h"

namespace wg {

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline bool valid_layout(int l) { return l == WG_NCHW || l == WG_NHWC; }
inline bool valid_mode(int m) { return m == WG_LOSSLESS || m == WG_SCALED; }
constexpr long long kIndexLimit = 0x7fffffffll;

// Shape checks shared by the convolution entry points, including the int32-exactness bound on
// the input channels.
inline int check_shape(int N, int C, int H, int W, int K) {
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0) return WG_EINVAL;
    if (C > WG_MAX_CHANNELS) return WG_EUNSUPPORTED;
    const long long hw = (long long)H * W;
    if (hw > kIndexLimit) return WG_EUNSUPPORTED;
    if ((long long)N * C > kIndexLimit / hw || (long long)N * K > kIndexLimit / hw) return WG_EUNSUPPORTED;
    if ((long long)K * C * 9 > kIndexLimit) return WG_EUNSUPPORTED;
    const long long tiles = (long long)N * ((H + 3) / 4) * ((W + 3) / 4);
    if (tiles + kTilePad > kIndexLimit / 64) return WG_EUNSUPPORTED;
    return WG_OK;
}

inline int check_filter_shape(int K, int C) {
    if (K <= 0 || C <= 0) return WG_EINVAL;
    if (C > WG_MAX_CHANNELS) return WG_EUNSUPPORTED;
    if ((long long)K * C * 9 > kIndexLimit) return WG_EUNSUPPORTED;
    return WG_OK;
}

inline int status_of(hipError_t e) { return e == hipSuccess ? WG_OK : WG_ERUNTIME; }

}  // namespace wg
