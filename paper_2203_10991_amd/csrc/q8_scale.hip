// Per-tensor scale and the activations' 8-bit cast of the 8-bit path (Sec. 5, 8-bit rows; the paper fixes no scale
// rule).  One power-of-two scale per tensor from its current maximum magnitude: the largest s = 2^e with
// s * max|t| <= top, e kept in [-126, 126] so that s and 1/s are normal numbers, s = 1 for an all-zero tensor or a
// maximum that is not finite.  The scale never visits the host: it is written to a 4-float record in device memory
//     rec[0] = s,  rec[1] = 1/s,  rec[2] = bit pattern of max|t|,  rec[3] = 0
// which the 8-bit prune, the cast below and the 8-bit update GEMM read there.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "nm_internal.h"

namespace nm {

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// (a fill kernel, not a memset: safe to record into a HIP graph)
__global__ void q8_scale_begin_kernel(float *rec)
{
    if (threadIdx.x < 4) ((uint32_t *)rec)[threadIdx.x] = 0u;
}

// max over the bit patterns of |t|: they order like the magnitudes, with infinity and every NaN on top.
// One thread = one 16-byte piece of a row per trip of a grid-stride loop; wave maximum, then one atomic per wave
// (the maximum does not depend on the order of the atomics: the result is reproducible).
template <int DT>
__global__ __launch_bounds__(256) void q8_amax_kernel(const void *__restrict__ t_, int64_t R, int64_t C, int64_t ld, float *rec)
{
    constexpr int VEC = DT == NM_DT_F32 ? 4 : 8, ESZ = DT == NM_DT_F32 ? 4 : 2;
    const int64_t cpr = C / VEC, n = R * cpr;
    uint32_t m = 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const int64_t r = i / cpr, c = (i - r * cpr) * VEC;
        const u32x4_t v = *(const u32x4_t *)((const char *)t_ + (r * ld + c) * ESZ);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (DT == NM_DT_F32) m = max(m, v[j] & 0x7fffffffu);
            else { m = max(m, (v[j] << 16) & 0x7fff0000u); m = max(m, v[j] & 0x7fff0000u); }
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, d));
    if ((threadIdx.x & 63) == 0 && m) atomicMax((uint32_t *)rec + 2, m);
}

__global__ void q8_scale_end_kernel(float *rec, float top)
{
    if (threadIdx.x != 0) return;
    const uint32_t mb = ((const uint32_t *)rec)[2];
    float s = 1.0f, inv = 1.0f;
    if (mb != 0 && mb < 0x7f800000u && top > 0.0f && top < __builtin_inff()) {
        int em, et;
        const float fm = frexpf(__uint_as_float(mb), &em), ft = frexpf(top, &et);     // x = f * 2^e, f in [0.5, 1)
        int e = et - em - (ft >= fm ? 0 : 1);                                          // largest e with 2^e * max <= top
        e = e > 126 ? 126 : e < -126 ? -126 : e;
        s = __uint_as_float((uint32_t)(127 + e) << 23);
        inv = __uint_as_float((uint32_t)(127 - e) << 23);
    }
    rec[0] = s;
    rec[1] = inv;
}

hipError_t launch_q8_scale(int dt, const void *t, int64_t R, int64_t C, int64_t ld, float top, float *rec, hipStream_t st)
{
    hipLaunchKernelGGL(q8_scale_begin_kernel, dim3(1), dim3(64), 0, st, rec);
    const int64_t pieces = R * (C / (dt == NM_DT_F32 ? 4 : 8));
    if (pieces > 0) {
        const int64_t blocks = std::min<int64_t>((pieces + 255) / 256, 256 * 16);
        if (dt == NM_DT_F32) hipLaunchKernelGGL(q8_amax_kernel<NM_DT_F32>, dim3((unsigned)blocks), dim3(256), 0, st, t, R, C, ld, rec);
        else hipLaunchKernelGGL(q8_amax_kernel<NM_DT_BF16>, dim3((unsigned)blocks), dim3(256), 0, st, t, R, C, ld, rec);
    }
    hipLaunchKernelGGL(q8_scale_end_kernel, dim3(1), dim3(64), 0, st, rec, top);
    return hipGetLastError();
}

// binary32 -> e4m3 (OCP), round to nearest even, magnitudes beyond 448 saturate: the hardware conversion after a
// clamp (it would otherwise produce the format's NaN where this cast saturates).  Four values per call pair.
__device__ __forceinline__ uint32_t pack4_e4m3(float a, float b, float c, float d)
{
    a = __builtin_amdgcn_fmed3f(a, -448.0f, 448.0f); b = __builtin_amdgcn_fmed3f(b, -448.0f, 448.0f);
    c = __builtin_amdgcn_fmed3f(c, -448.0f, 448.0f); d = __builtin_amdgcn_fmed3f(d, -448.0f, 448.0f);
    int w = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, w, true);
    return (uint32_t)w;
}

// one thread = 16 consecutive elements of a row -> one 16-byte store
template <int DT>
__global__ __launch_bounds__(256) void cast_e4m3_kernel(const void *__restrict__ h_, int64_t R, int64_t C, int64_t ld,
                                                       const float *__restrict__ rec, uint8_t *__restrict__ h8, int64_t ld8)
{
    const int64_t cpr = C / 16, i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= R * cpr) return;
    const int64_t r = i / cpr, c = (i - r * cpr) * 16;
    const float s = rec[0];
    float x[16];
    if constexpr (DT == NM_DT_F32) {
        const float4 *src = (const float4 *)((const float *)h_ + r * ld + c);
#pragma unroll
        for (int j = 0; j < 4; ++j) { const float4 v = src[j]; x[4 * j] = v.x; x[4 * j + 1] = v.y; x[4 * j + 2] = v.z; x[4 * j + 3] = v.w; }
    } else {
        const u32x4_t *src = (const u32x4_t *)((const uint16_t *)h_ + r * ld + c);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const u32x4_t v = src[j];
#pragma unroll
            for (int k = 0; k < 4; ++k) { x[8 * j + 2 * k] = __uint_as_float(v[k] << 16); x[8 * j + 2 * k + 1] = __uint_as_float(v[k] & 0xffff0000u); }
        }
    }
    u32x4_t o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = pack4_e4m3(x[4 * j] * s, x[4 * j + 1] * s, x[4 * j + 2] * s, x[4 * j + 3] * s);
    *(u32x4_t *)(h8 + r * ld8 + c) = o;
}

hipError_t launch_cast_e4m3(int dt, const void *h, int64_t R, int64_t C, int64_t ld, const float *rec, uint8_t *h8, int64_t ld8,
                            hipStream_t st)
{
    const int64_t threads = R * (C / 16);
    if (threads == 0) return hipSuccess;
    const int64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffll) return hipErrorInvalidConfiguration;
    if (dt == NM_DT_F32) hipLaunchKernelGGL(cast_e4m3_kernel<NM_DT_F32>, dim3((unsigned)blocks), dim3(256), 0, st, h, R, C, ld, rec, h8, ld8);
    else hipLaunchKernelGGL(cast_e4m3_kernel<NM_DT_BF16>, dim3((unsigned)blocks), dim3(256), 0, st, h, R, C, ld, rec, h8, ld8);
    return hipGetLastError();
}

}  // namespace nm
