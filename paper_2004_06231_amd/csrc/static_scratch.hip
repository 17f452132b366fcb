// A fixed arena in device memory for callers that must not allocate (einet_logp_static): the activations of one
// forward pass live here instead of in a caller-provided workspace.  Every GPU the library runs on holds its own
// copy of the array, at its own address, until the process ends.
#include "kernels.hpp"

#include <mutex>

namespace einet_impl {

namespace {

static __device__ __align__(256) unsigned char scratch[EINET_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices] = {nullptr};   // device address of `scratch` on device d, once asked for

}  // namespace

// Device address of the arena on the current device.  In host code the array's name is only a handle for the
// symbol, not an address a kernel could use, so the address is asked for once per device (with that device
// current) and kept.
hipError_t static_scratch_address(void** ptr) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(g_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace einet_impl
