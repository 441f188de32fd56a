// Scratch memory that exists without any allocation call: a file-scope device
// array, one copy per GPU, held until the process ends. It serves the entry
// point for callers that cannot allocate (code under HIP graph capture, serving
// loops, harnesses that forbid hipMalloc): segmented_decode_step_static.
//
// In host code the array's name is only a stand-in for the symbol; the device
// address is asked for once per device with hipGetSymbolAddress, with that
// device current, and kept. Everything on the host side uses that address.
#include <hip/hip_runtime.h>

#include <mutex>

#include "en_internal.h"

static __device__ __align__(256) unsigned char scratch[EN_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_lock;
void *g_ptr[MAX_DEVICES] = {};       // device address of `scratch` on each device, null: not asked for yet
}

// Device address of the current device's copy of the static scratch. The first
// call on a device asks the runtime for it (no allocation: the array is part of
// the loaded code object); later calls return the kept address.
int en_static_scratch(void **ptr_out, size_t *bytes_out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return (int)e;
    if (dev < 0 || dev >= MAX_DEVICES)
        return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess)
            return (int)e;
        if (!p)
            return (int)hipErrorInvalidSymbol;
        g_ptr[dev] = p;
    }
    *ptr_out = g_ptr[dev];
    *bytes_out = EN_STATIC_SCRATCH_BYTES;
    return 0;
}
