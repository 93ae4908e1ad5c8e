// Device memory that exists without any allocation call: a fixed array in the library's code
// object, for the entry point that serves callers who may not allocate (ens_predict_static).
// Every GPU the library runs on holds its own copy of the array, at its own address, from the
// moment the code object is loaded there until the process ends.
#include <hip/hip_runtime.h>

#include <mutex>

#include "static_scratch.h"

namespace ens {

// Host code must never use this name as an address: here it is only the handle that
// hipGetSymbolAddress resolves, per device, into the array's device address.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_lock;
void* g_ptr[MAX_DEVICES];      // the array's address on each device, resolved on first use there
}  // namespace

hipError_t static_scratch(void** ptr, size_t* bytes) {
    if (!ptr || !bytes) return hipErrorInvalidValue;
    *ptr = nullptr;
    *bytes = 0;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));    // the current device's copy
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_ptr[dev] = p;
    }
    *ptr = g_ptr[dev];
    *bytes = STATIC_SCRATCH_BYTES;
    return hipSuccess;
}

}  // namespace ens
