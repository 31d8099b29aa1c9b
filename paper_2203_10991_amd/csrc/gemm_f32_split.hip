// Update GEMM (eq. (3)) for binary32 operands on the SPARSE 16-bit matrix path.
//
// gfx950 has no sparse (and no fast) binary32 matrix instruction: the dense fp32 MFMA path executes every product at
// 157 TFLOP/s.  Here each binary32 value x is written as a sum of three bf16 terms,
//     x0 = bf16(x),  x1 = bf16(x - x0),  x2 = bf16(x - x0 - x1)          (round to nearest even; both differences are
// exact in binary32), which carries 24 significant bits, and the product of the compressed operand a and the
// activations b is formed from the six partial products whose terms have i + j <= 2:
//     a b ~ a0 b0 + (a0 b1 + a1 b0) + (a0 b2 + a1 b1 + a2 b0).
// The three dropped products are below 2^-24 |a b|.  The update GEMM reduces over tokens, so the six products are ONE
// run of the 16-bit sparse update GEMM over operands stacked along the token axis: six segments of T tokens each,
// segment k holding the planes of term k (the compressed operand's planes share its index words, which are copied once
// per segment), smallest terms first, all accumulated in binary32 in the same accumulation registers.  Six times the
// 16-bit sparse work costs less than half of one dense fp32 GEMM.
//
// Non-finite inputs: the first plane carries the infinity or NaN, the other two are zero; the results they touch are
// non-finite, though an infinity may come out as a NaN (infinity times a zero low-order term).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"

namespace nm {

namespace {

__device__ __forceinline__ uint32_t bf16_rne_bits(float x)          // finite or not: NaN stays NaN (quiet bit kept)
{
    const uint32_t b = __float_as_uint(x);
    if ((b & 0x7fffffffu) > 0x7f800000u) return (b >> 16) | 0x40u;
    return (b + 0x7fffu + ((b >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ void split3(float x, uint32_t &p0, uint32_t &p1, uint32_t &p2)
{
    p0 = bf16_rne_bits(x);
    const float x0 = __uint_as_float(p0 << 16);
    const bool finite = (__float_as_uint(x0) & 0x7f800000u) != 0x7f800000u;
    const float r1 = finite ? x - x0 : 0.f;
    p1 = bf16_rne_bits(r1);
    const float r2 = r1 - __uint_as_float(p1 << 16);
    p2 = bf16_rne_bits(r2);
}

// Which of the three planes each of the six segments of a stacked operand holds: segment k of the compressed operand is
// plane TERM_A[k], segment k of the activations plane TERM_B[k]; smallest products first.
struct SplitDst { uint16_t *seg[6]; int plane[6]; };
constexpr int TERM_A[6] = {2, 1, 0, 1, 0, 0}, TERM_B[6] = {0, 1, 2, 0, 1, 0};

// x: rows x cols binary32 (row stride ld, cols % 4 == 0) -> six contiguous rows x cols bf16 segments, segment k
// holding plane dst.plane[k] of x
__global__ __launch_bounds__(256) void split3_bf16_kernel(const float *__restrict__ x, int64_t rows, int64_t cols, int64_t ld,
                                                          SplitDst dst)
{
    const int64_t c4 = cols / 4;
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= rows * c4) return;
    const int64_t r = n / c4, c = (n - r * c4) * 4;
    const float4 v = *(const float4 *)(x + r * ld + c);
    uint32_t p[3][4];
    split3(v.x, p[0][0], p[1][0], p[2][0]);
    split3(v.y, p[0][1], p[1][1], p[2][1]);
    split3(v.z, p[0][2], p[1][2], p[2][2]);
    split3(v.w, p[0][3], p[1][3], p[2][3]);
    uint2 w[3];
#pragma unroll
    for (int i = 0; i < 3; ++i) w[i] = make_uint2(p[i][0] | (p[i][1] << 16), p[i][2] | (p[i][3] << 16));
    const int64_t o = r * cols + c;
#pragma unroll
    for (int k = 0; k < 6; ++k) {
        const int i = dst.plane[k];
        *(uint2 *)(dst.seg[k] + o) = i == 0 ? w[0] : (i == 1 ? w[1] : w[2]);
    }
}

// n 16-byte words of src, `copies` times one after the other into dst
__global__ __launch_bounds__(256) void replicate_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int64_t n, int copies)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const uint4 v = src[i];
    for (int k = 0; k < copies; ++k) dst[(int64_t)k * n + i] = v;
}

inline size_t round256(size_t b) { return (b + 255) / 256 * 256; }

}  // namespace

// workspace layout: [6 segments of vals][6 segments of h][6 copies of meta][workspace of the 16-bit GEMM over 6T tokens],
// each part on a 256-byte boundary
size_t update_gemm_f32_split_workspace(int64_t T, int64_t O, int64_t I)
{
    if (T <= 0 || O <= 0 || I <= 0) return 0;
    return round256(6 * (size_t)(T / 2) * O * 2) + round256(6 * (size_t)T * I * 2) + round256(6 * (size_t)(T / 16) * O * 2) +
           round256(update_gemm_smfmac_workspace(6 * T, O, I));
}

hipError_t launch_update_gemm_f32_split(const void *vals, const uint16_t *meta, const void *h, int64_t ldh, float *dW,
                                        int64_t lddw, int64_t T, int64_t O, int64_t I, float beta, void *workspace,
                                        hipStream_t st)
{
    if (O == 0 || I == 0) return hipSuccess;
    if (T == 0) return launch_update_gemm_smfmac(nullptr, meta, nullptr, I, dW, lddw, 0, O, I, beta, nullptr, st);
    char *w = (char *)workspace;
    const int64_t a_elems = (T / 2) * O, b_elems = T * I, m_bytes = (T / 16) * O * 2;
    uint16_t *a = (uint16_t *)w;
    uint16_t *b = (uint16_t *)(w + round256(6 * (size_t)a_elems * 2));
    uint16_t *m = (uint16_t *)((char *)b + round256(6 * (size_t)b_elems * 2));
    void *gemm_ws = (char *)m + round256(6 * (size_t)m_bytes);
    SplitDst da, db;
    for (int k = 0; k < 6; ++k) {
        da.seg[k] = a + k * a_elems; da.plane[k] = TERM_A[k];
        db.seg[k] = b + k * b_elems; db.plane[k] = TERM_B[k];
    }
    const int64_t na = a_elems / 4, nb = T * (I / 4), nm16 = m_bytes / 16;
    if ((na + 255) / 256 > 0x7fffffffll || (nb + 255) / 256 > 0x7fffffffll) return hipErrorInvalidConfiguration;   // one thread per 4 values
    hipLaunchKernelGGL(split3_bf16_kernel, dim3((unsigned)((na + 255) / 256)), dim3(256), 0, st, (const float *)vals,
                       (int64_t)1, a_elems, a_elems, da);
    hipLaunchKernelGGL(split3_bf16_kernel, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, st, (const float *)h, T, I, ldh, db);
    hipLaunchKernelGGL(replicate_kernel, dim3((unsigned)((nm16 + 255) / 256)), dim3(256), 0, st, (const uint4 *)meta, (uint4 *)m,
                       nm16, 6);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // one run over the stacked operands: the reduction over 6T tokens sums the six products, in the order of the segments
    return launch_update_gemm_smfmac(a, m, b, I, dW, lddw, 6 * T, O, I, beta, gemm_ws, st);
}

}  // namespace nm
