// The library's own scratch memory, for the one entry point that must not allocate
// (anr_conv2d_noalloc): a fixed array in device memory that every GPU the library runs on
// holds from the moment the code object is loaded until the process ends.
#include "anr_kernels.h"

namespace anr {
namespace {

// In host code this name is only a handle for hipGetSymbolAddress: it is not a device address
// and must never be handed to a kernel or a runtime call as one.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];   // per device: each GPU has its own copy of the array

}  // namespace

// Device address of the current device's copy of the array.  The first call on a device asks
// the runtime for it (no allocation: the array came with the code object); later calls read
// the cached pointer.  Two threads racing on the first call both get the same answer.
hipError_t static_scratch(void** ptr, size_t* bytes)
{
    *ptr = nullptr;
    *bytes = 0;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *ptr = p;
    *bytes = kStaticScratchBytes;
    return hipSuccess;
}

}  // namespace anr
