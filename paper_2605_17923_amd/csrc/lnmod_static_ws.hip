// lnmod_static_ws.hip -- the device array behind lnmod_backward_static, the backward entry point
// that allocates nothing, and the look-up of its address.  Linked into the operator library only.
#include <hip/hip_runtime.h>

#include <atomic>

#include "lnmod_launch.hpp"

namespace lnmod {

// One array per GPU, held from the time the library's code is loaded on that GPU until the
// process ends.  In host code the name below is only a handle: the device address comes from
// hipGetSymbolAddress, once per device, and that address is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];

hipError_t static_workspace(float** ptr) {
    constexpr int kMaxDevices = 64;
    static std::atomic<void*> address[kMaxDevices];          // zero-initialised: not looked up yet
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void* p = address[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        // two threads may both get here; they obtain the same address
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        address[dev].store(p, std::memory_order_release);
    }
    *ptr = static_cast<float*>(p);
    return hipSuccess;
}

}  // namespace lnmod
