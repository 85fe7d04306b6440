// Device memory that belongs to the library itself: one file-scope array per GPU, for the entry point
// that must not allocate (esrnn_predict_static).  Host code never uses the array's name as an address:
// the name is a host-side handle, and the device address is asked for once per device with
// hipGetSymbolAddress while that device is current, then kept.
#include <mutex>

#include "esrnn_internal.h"

namespace esrnn {

namespace {

static __device__ __align__(256) unsigned char scratch[ESRNN_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU; null until first asked for

}  // namespace

hipError_t static_scratch(void **ptr, size_t *bytes)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        // every GPU holds its own copy of the array at its own address
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    *bytes = ESRNN_STATIC_SCRATCH_BYTES;
    return hipSuccess;
}

}  // namespace esrnn
