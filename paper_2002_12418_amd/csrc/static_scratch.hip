// The one device buffer the library owns without ever allocating it: a fixed array in the code object, for the
// entry point that serves callers which cannot allocate device memory (mnn_conv_run_static).
//
// The array's name is a host-side stand-in, not a device address; the address on a device comes from
// hipGetSymbolAddress, asked once per device with that device current and kept.  Host code uses that pointer only.
#include <hip/hip_runtime.h>
#include <mutex>
#include "kernels.hpp"

namespace mnnconv {
namespace {

constexpr size_t kScratchFloats = kStaticScratchBytes / sizeof(float);
static __device__ __attribute__((used)) __align__(256) float scratch[kScratchFloats];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
float* g_ptr[kMaxDevices] = {};

}  // namespace

hipError_t static_scratch(float** ptr)
{
    if (!ptr) return hipErrorInvalidValue;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));     // this device's copy of the array
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_ptr[dev] = static_cast<float*>(p);
    }
    *ptr = g_ptr[dev];
    return hipSuccess;
}

}  // namespace mnnconv
