// Measurement aid, not part of the method: a streaming kernel with the read:write mix of the 16-bit prune + compress
// (16 bytes read for every 9 written: the gradient in, kept values and index words out) and fully contiguous
// instructions, so that a benchmark can state what this mix reaches on the device next to the prune kernel's own
// rate.  A workgroup of 256 threads reads 16 rows of 4 KB and writes 9: thread t reads the 16-byte words
// src[(16 b + r) * 256 + t], r = 0..15, and writes dst[(9 b + k) * 256 + t] = src word k XOR src word k + 7, k = 0..8
// (every word read is used, nothing can be dropped by the compiler).  Loads and stores are the streaming (non-temporal)
// forms, as in the prune kernels: with both, this mix measures 9 % faster on the device than with plain ones (5.75
// against 5.24 TB/s; either alone gives 1-2 %).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"

namespace nm {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void rw_mix_probe_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int64_t n_blocks)
{
    const int64_t b = blockIdx.x;
    if (b >= n_blocks) return;
    const u32x4_t *s = (const u32x4_t *)(src + b * 16 * 256 + threadIdx.x);
    u32x4_t in[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) in[r] = __builtin_nontemporal_load(s + r * 256);
    u32x4_t *d = (u32x4_t *)(dst + b * 9 * 256 + threadIdx.x);
#pragma unroll
    for (int k = 0; k < 9; ++k) __builtin_nontemporal_store(in[k] ^ in[k + 7], d + k * 256);
}

hipError_t launch_rw_mix_probe(const void *src, void *dst, int64_t n_blocks, hipStream_t st)
{
    if (n_blocks == 0) return hipSuccess;
    if (n_blocks > 0x7fffffffll) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(rw_mix_probe_kernel, dim3((unsigned)n_blocks), dim3(256), 0, st, (const uint4 *)src, (uint4 *)dst, n_blocks);
    return hipGetLastError();
}

}  // namespace nm
