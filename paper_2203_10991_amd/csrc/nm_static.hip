// Static device scratch for callers that cannot allocate (code under HIP graph capture, serving loops, harnesses
// that forbid hipMalloc): nm_update_gemm_static takes the split-K partial sums' buffer from this array instead of a
// caller's workspace.  Every GPU the library runs on holds its own copy of the array, at its own address, until the
// process ends; all calls on a GPU share it, so calls that overlap in time on one GPU race.  The split-K kernels
// write every partial sum they later read, so nothing in the array has to start at zero.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "nm_internal.h"

namespace nm {

constexpr size_t STATIC_SCRATCH_BYTES = (size_t)64 << 20;       // 64 MiB per GPU
constexpr int MAX_DEVICES = 64;

// In host code this name is a stand-in for the symbol, not a device address: it is only ever used inside HIP_SYMBOL().
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

static std::mutex g_lock;
static void *g_ptr[MAX_DEVICES];           // device address of `scratch` on each device, once looked up

size_t static_scratch_bytes() { return STATIC_SCRATCH_BYTES; }

hipError_t static_scratch(void **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(g_lock);
    if (!g_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));      // the current device's copy
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_ptr[dev] = p;
    }
    *ptr = g_ptr[dev];
    return hipSuccess;
}

}  // namespace nm
