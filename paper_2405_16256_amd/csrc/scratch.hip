// Device memory that belongs to the library itself: one fixed array per GPU, used as the forward pass's scratch by
// the entry point that may not allocate.  The array's name is a host-side handle only; its device address is looked
// up once per device and that pointer is what kernels, and every other piece of host code, receive.
#include <hip/hip_runtime.h>

#include <stddef.h>

#include "kernels.h"

namespace hh {

static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES];   // per device: address of that device's copy of `scratch` (null: not looked up yet)
}  // namespace

// Looks up this device's copy of the array.  `device` must be the current device.  Called from context creation.
hipError_t static_scratch_init(int device) {
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    if (g_scratch_ptr[device]) return hipSuccess;
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = p;
    return hipSuccess;
}

// Device address of the array on `device`, or null before static_scratch_init(device) has succeeded.
void* static_scratch(int device) {
    return device >= 0 && device < MAX_DEVICES ? g_scratch_ptr[device] : nullptr;
}

}  // namespace hh
