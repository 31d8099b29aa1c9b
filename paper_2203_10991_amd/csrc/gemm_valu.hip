// Update GEMM, eq. (3):  dW[O x I] = beta*dW + decompress(vals, meta)^T h.
//
// Vector-ALU tile kernel (binary32 multiply-add, no matrix instruction).  It serves the
// NM_F32 dtype, for which gfx950 has no sparse matrix instruction, and shapes the MFMA
// kernels do not cover.  A 64x64 output tile per 256-thread workgroup; the reduction axis is
// walked one 16-token group at a time: the group's kept values are expanded to dense rows in
// LDS by the index words, h rows are staged beside them, each thread owns a 4x4 micro-tile.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"

namespace nm {

template <int DT> __device__ __forceinline__ float ld_elem(const void *p, int64_t i);
template <> __device__ __forceinline__ float ld_elem<NM_DT_F32>(const void *p, int64_t i) { return ((const float *)p)[i]; }
template <> __device__ __forceinline__ float ld_elem<NM_DT_BF16>(const void *p, int64_t i)
{
    return __uint_as_float((uint32_t)((const uint16_t *)p)[i] << 16);
}

template <int DT>
__global__ __launch_bounds__(256) void update_gemm_valu_kernel(
    const void *__restrict__ vals, const uint16_t *__restrict__ meta, const void *__restrict__ h, int64_t ldh,
    float *__restrict__ dW, int64_t lddw, int64_t n_groups, int64_t O, int64_t I, float beta)
{
    __shared__ float As[16][64 + 4];     // dense rows of the sparse operand: [token in group][o]
    __shared__ float Bs[16][64 + 4];     // h rows: [token in group][i]
    const int tid = threadIdx.x;
    const int64_t o0 = (int64_t)blockIdx.y * 64, i0 = (int64_t)blockIdx.x * 64;
    const int ty = tid / 16, tx = tid % 16;           // micro-tile rows 4*ty.., cols 4*tx..
    float acc[4][4] = {};

    for (int64_t G = 0; G < n_groups; ++G) {
        // expand: 4 threads per column, one quad each
        {
            const int c = tid >> 2, q = tid & 3;
            const int64_t o = o0 + c;
            float x[4] = {0.f, 0.f, 0.f, 0.f};
            if (o < O) {
                const uint32_t nib = ((uint32_t)meta[G * O + o] >> (4 * q)) & 0xfu;
                const float v0 = ld_elem<DT>(vals, (G * O + o) * 8 + 2 * q);
                const float v1 = ld_elem<DT>(vals, (G * O + o) * 8 + 2 * q + 1);
                x[nib & 3u] = v0;
                x[nib >> 2] = v1;
            }
#pragma unroll
            for (int p = 0; p < 4; ++p) As[4 * q + p][c] = x[p];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + 256 * e, r = idx >> 6, c = idx & 63;
            const int64_t i = i0 + c;
            Bs[r][c] = i < I ? ld_elem<DT>(h, (G * 16 + r) * ldh + i) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) { a[j] = As[k][4 * ty + j]; b[j] = Bs[k][4 * tx + j]; }
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[r][c] = fmaf(a[r], b[c], acc[r][c]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t o = o0 + 4 * ty + r;
        if (o >= O) continue;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int64_t i = i0 + 4 * tx + c;
            if (i >= I) continue;
            float *p = dW + o * lddw + i;
            *p = beta != 0.f ? (beta * *p + acc[r][c]) : acc[r][c];
        }
    }
}

hipError_t launch_update_gemm_valu(int dt, const void *vals, const uint16_t *meta, const void *h, int64_t ldh,
                                   float *dW, int64_t lddw, int64_t T, int64_t O, int64_t I, float beta, hipStream_t st)
{
    if (O == 0 || I == 0) return hipSuccess;
    dim3 grid((unsigned)((I + 63) / 64), (unsigned)((O + 63) / 64));
    if (dt == NM_DT_F32)
        hipLaunchKernelGGL(update_gemm_valu_kernel<NM_DT_F32>, grid, dim3(256), 0, st, vals, meta, h, ldh, dW, lddw,
                           T / 16, O, I, beta);
    else
        hipLaunchKernelGGL(update_gemm_valu_kernel<NM_DT_BF16>, grid, dim3(256), 0, st, vals, meta, h, ldh, dW, lddw,
                           T / 16, O, I, beta);
    return hipGetLastError();
}

}  // namespace nm
