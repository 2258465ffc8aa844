// Scratch memory of the library's own, for the one entry point that must not allocate
// (cf_step_fused_static): a file-scope device array, one copy per GPU, held until the process ends.
//
// In host code the array's name is only a stand-in: its device address is asked for once per
// device, with that device current, and kept; every kernel takes that address as an argument.
#include <hip/hip_runtime.h>

#include "cf_internal.h"

namespace cf {
namespace {

static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];       // per device: each GPU holds its own copy at its own address

}  // namespace

hipError_t static_scratch(void **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace cf
