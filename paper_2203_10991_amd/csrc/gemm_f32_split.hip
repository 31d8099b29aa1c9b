// Update GEMM (eq. (3)) for binary32 operands on the SPARSE 16-bit matrix path.
//
// gfx950 has no sparse (and no fast) binary32 matrix instruction: the dense fp32 MFMA path executes every product at
// 157 TFLOP/s.  Here each binary32 value x is written as a sum of three bf16 terms,
//     x0 = bf16(x),  x1 = bf16(x - x0),  x2 = bf16(x - x0 - x1)          (round to nearest even; both differences are
// exact in binary32), which carries 24 significant bits, and the product of the compressed operand a and the
// activations b is formed from the six partial products whose terms have i + j <= 2:
//     a b ~ a0 b0 + (a0 b1 + a1 b0) + (a0 b2 + a1 b1 + a2 b0).
// The three dropped products are below 2^-24 |a b|.  Each partial product is one run of the 16-bit sparse update GEMM
// (the three planes of the compressed operand share its index words), accumulated into dW in binary32, smallest
// terms first.  Six sparse 16-bit GEMMs cost less than half of one dense fp32 GEMM.
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

// x: rows x cols binary32 (row stride ld, cols % 4 == 0) -> three contiguous rows x cols bf16 planes
__global__ __launch_bounds__(256) void split3_bf16_kernel(const float *__restrict__ x, int64_t rows, int64_t cols, int64_t ld,
                                                          uint16_t *__restrict__ p0, uint16_t *__restrict__ p1,
                                                          uint16_t *__restrict__ p2)
{
    const int64_t c4 = cols / 4;
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= rows * c4) return;
    const int64_t r = n / c4, c = (n - r * c4) * 4;
    const float4 v = *(const float4 *)(x + r * ld + c);
    uint32_t a[4], b[4], d[4];
    split3(v.x, a[0], b[0], d[0]);
    split3(v.y, a[1], b[1], d[1]);
    split3(v.z, a[2], b[2], d[2]);
    split3(v.w, a[3], b[3], d[3]);
    const int64_t o = r * cols + c;
    *(uint2 *)(p0 + o) = make_uint2(a[0] | (a[1] << 16), a[2] | (a[3] << 16));
    *(uint2 *)(p1 + o) = make_uint2(b[0] | (b[1] << 16), b[2] | (b[3] << 16));
    *(uint2 *)(p2 + o) = make_uint2(d[0] | (d[1] << 16), d[2] | (d[3] << 16));
}

inline size_t round256(size_t b) { return (b + 255) / 256 * 256; }

}  // namespace

// workspace layout: [3 planes of vals][3 planes of h][workspace of the 16-bit GEMM], each part on a 256-byte boundary
size_t update_gemm_f32_split_workspace(int64_t T, int64_t O, int64_t I)
{
    if (T <= 0 || O <= 0 || I <= 0) return 0;
    return 3 * round256((size_t)(T / 2) * O * 2) + 3 * round256((size_t)T * I * 2) + round256(update_gemm_smfmac_workspace(T, O, I));
}

hipError_t launch_update_gemm_f32_split(const void *vals, const uint16_t *meta, const void *h, int64_t ldh, float *dW,
                                        int64_t lddw, int64_t T, int64_t O, int64_t I, float beta, void *workspace,
                                        hipStream_t st)
{
    if (O == 0 || I == 0) return hipSuccess;
    if (T == 0) return launch_update_gemm_smfmac(nullptr, meta, nullptr, I, dW, lddw, 0, O, I, beta, nullptr, st);
    char *w = (char *)workspace;
    const size_t a_bytes = round256((size_t)(T / 2) * O * 2), b_bytes = round256((size_t)T * I * 2);
    uint16_t *a[3], *b[3];
    for (int i = 0; i < 3; ++i) a[i] = (uint16_t *)(w + i * a_bytes);
    for (int i = 0; i < 3; ++i) b[i] = (uint16_t *)(w + 3 * a_bytes + i * b_bytes);
    void *gemm_ws = w + 3 * a_bytes + 3 * b_bytes;

    const int64_t na = (T / 2) * O / 4, nb = T * (I / 4);
    hipLaunchKernelGGL(split3_bf16_kernel, dim3((unsigned)((na + 255) / 256)), dim3(256), 0, st, (const float *)vals,
                       (int64_t)1, (T / 2) * O, (T / 2) * O, a[0], a[1], a[2]);
    hipLaunchKernelGGL(split3_bf16_kernel, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, st, (const float *)h, T, I, ldh,
                       b[0], b[1], b[2]);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // smallest terms first; the first run applies the caller's beta, the others add
    static const int term[6][2] = {{2, 0}, {1, 1}, {0, 2}, {1, 0}, {0, 1}, {0, 0}};
    for (int k = 0; k < 6; ++k) {
        e = launch_update_gemm_smfmac(a[term[k][0]], meta, b[term[k][1]], I, dW, lddw, T, O, I, k == 0 ? beta : 1.0f, gemm_ws, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace nm
