// Device scratch that belongs to the library itself: a fixed array in the code object, for the one entry point
// that may not allocate (race_attn_fwd_static).  Every GPU the library runs on holds its own copy of the array
// from the moment the code object is loaded there until the process ends.
#include <hip/hip_runtime.h>

#include <mutex>

#include "internal.h"

namespace race {

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];       // device address of `scratch` on device i (null: not asked for yet)
}  // namespace

// Address of the current device's copy of the array.  The array's name is only a handle on the host: its device
// address is looked up once per device, with that device current, and remembered.
hipError_t static_scratch(void **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
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

}  // namespace race
