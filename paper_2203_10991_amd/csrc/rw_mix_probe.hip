// Measurement aid, not part of the method: a streaming kernel with the read:write mix of the 16-bit prune + compress
// (16 bytes read for every 9 written: the gradient in, kept values and index words out) and fully contiguous
// instructions, so that a benchmark can state what this mix reaches on the device next to the prune kernel's own
// rate.  A workgroup of 256 threads reads 16 rows of 4 KB and writes 9: thread t reads the 16-byte words
// src[(16 b + r) * 256 + t], r = 0..15, and writes dst[(9 b + k) * 256 + t] = src word k XOR src word k + 7, k = 0..8
// (every word read is used, nothing can be dropped by the compiler).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"

namespace nm {

__global__ __launch_bounds__(256) void rw_mix_probe_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int64_t n_blocks)
{
    const int64_t b = blockIdx.x;
    if (b >= n_blocks) return;
    const uint4 *s = src + b * 16 * 256 + threadIdx.x;
    uint4 in[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) in[r] = s[r * 256];
    uint4 *d = dst + b * 9 * 256 + threadIdx.x;
#pragma unroll
    for (int k = 0; k < 9; ++k)
        d[k * 256] = make_uint4(in[k].x ^ in[k + 7].x, in[k].y ^ in[k + 7].y, in[k].z ^ in[k + 7].z, in[k].w ^ in[k + 7].w);
}

hipError_t launch_rw_mix_probe(const void *src, void *dst, int64_t n_blocks, hipStream_t st)
{
    if (n_blocks == 0) return hipSuccess;
    if (n_blocks > 0x7fffffffll) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(rw_mix_probe_kernel, dim3((unsigned)n_blocks), dim3(256), 0, st, (const uint4 *)src, (uint4 *)dst, n_blocks);
    return hipGetLastError();
}

}  // namespace nm
