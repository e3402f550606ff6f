// Split-K accumulators in a file-scope device array, for callers that must not allocate (HIP graph
// capture, serving loops, harnesses that forbid hipMalloc): bcq_gemv_noalloc uses this array where
// bcq_gemv takes a caller-provided workspace.
//
// Each GPU the library runs on holds its own copy of the array, at its own address, until the
// process ends.  In host code the array's name is only a handle for the runtime, not a device
// address: the address is asked from the runtime once per device (hipGetSymbolAddress, with that
// device current) and that pointer -- never the name -- is what kernels and fills receive.
#include <mutex>

#include "bcq_internal.h"

namespace bcq {

// One 64-bit accumulator word per padded output row (batch 1).
static __device__ __align__(256) unsigned long long scratch[kStaticScratchRows];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_lock;
void *g_scratch_ptr[kMaxDevices];  // per device: address of that device's copy, nullptr until asked
}  // namespace

hipError_t static_scratch(void **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(g_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // the current device's copy
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace bcq
