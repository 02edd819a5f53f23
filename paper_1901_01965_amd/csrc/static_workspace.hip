// winograd_conv2d_int8_static_workspace: the staged pipeline of winograd_conv2d_int8 through a
// scratch buffer that lives in the library, for callers that cannot allocate device memory
// (code under HIP graph capture, serving loops, harnesses that forbid it).
//
// `scratch` is one array per device that loads this library, held until the process ends.  In host
// code its name is not a device address, only a handle: hipGetSymbolAddress turns it into the
// array's address on the device that is current, once per device, and from then on only that
// address is used (kernel arguments).  Nothing here calls hipMalloc, hipFree or an allocating
// library routine.
#include <mutex>

#include "api_checks.h"

using namespace wg;

namespace {

constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
constexpr int kMaxDevices = 64;

}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// The array's address on the current device, asked from the runtime once per device (under a
// lock); nullptr if the runtime refuses.
unsigned char* static_scratch() {
    static std::mutex lock;
    static unsigned char* address[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> guard(lock);
    if (address[dev] == nullptr) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return nullptr;
        address[dev] = static_cast<unsigned char*>(ptr);
    }
    return address[dev];
}

}  // namespace

extern "C" {

size_t winograd_static_workspace_limit(void) { return kStaticScratchBytes; }

int winograd_conv2d_int8_static_workspace(const int8_t* x_dev, const void* packed_dev, int32_t* y_dev, int N, int C,
                                          int H, int W, int K, int layout, int mode, void* hip_stream) {
    if (!x_dev || !packed_dev || !y_dev || !valid_layout(layout) || !valid_mode(mode)) return WG_EINVAL;
    if (int st = check_shape(N, C, H, W, K)) return st;
    if (!aligned(x_dev, 4) || !aligned(y_dev, 4) || !aligned(packed_dev, 256)) return WG_EINVAL;
    const Problem p = make_problem(N, C, H, W, K);
    const WorkspaceLayout wl = workspace_layout(p, mode);
    if (wl.total > kStaticScratchBytes) return WG_ESMALLBUF;   // needs more scratch than the library holds
    unsigned char* const ws = static_scratch();
    if (ws == nullptr) return WG_ERUNTIME;
    // Nothing has to be cleared between calls: every value that reaches y was written earlier in this
    // call.  The contraction also reads the operand rows of the padding tiles (T rounded up to a
    // multiple of 64), which hold whatever the last call left there; those are integers that only
    // enter the accumulators of the same padding tiles, and the output transform never reads them.
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int8_t* V = reinterpret_cast<int8_t*>(ws + wl.v_off);
    int32_t* M = reinterpret_cast<int32_t*>(ws + wl.m_off);
    if (int st = status_of(launch_input_transform(x_dev, p, layout, mode, V, s))) return st;
    if (int st = status_of(launch_contraction(V, packed_dev, M, p, mode, s))) return st;
    return status_of(launch_output_transform(M, packed_dev, y_dev, p, layout, mode, s));
}

}  // extern "C"
