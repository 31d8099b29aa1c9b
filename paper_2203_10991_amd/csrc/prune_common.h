// Device helpers shared by the prune kernels: the counter-based random source, element access inside a 16-byte
// row vector, bf16 rounding.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"

namespace nm {

// ------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  Key words are wave-uniform (scalar registers).
// ------------------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// The same function for a call whose counter words 1-3 are wave-uniform, like the key (the high half of the call
// index, the stream and the domain word: only the low half of the call index differs between lanes).  Then half of
// the generator's first iteration, a multiply and an xor of its second and an xor of its third are scalar work; the
// result is the same word for word.
__device__ __forceinline__ void philox4x32_10_uniform_c123(uint32_t c0, uint32_t c1u, uint32_t c2u, uint32_t c3u,
                                                           uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    // first of the ten iterations: c1, c2, c3 uniform
    const uint64_t q1 = (uint64_t)M1 * c2u;                             // scalar
    const uint32_t a0 = (uint32_t)(q1 >> 32) ^ c1u ^ k0;                // scalar
    const uint32_t a1 = (uint32_t)q1;                                   // scalar
    const uint64_t q0 = (uint64_t)M0 * c0;
    const uint32_t a2 = (uint32_t)(q0 >> 32) ^ (c3u ^ k1);
    const uint32_t a3 = (uint32_t)q0;
    k0 += W0; k1 += W1;
    // second iteration: c0, c1 uniform
    const uint64_t r0 = (uint64_t)M0 * a0;                              // scalar
    const uint64_t r1 = (uint64_t)M1 * a2;
    const uint32_t b0 = (uint32_t)(r1 >> 32) ^ (a1 ^ k0);
    const uint32_t b1 = (uint32_t)r1;
    const uint32_t b2 = a3 ^ ((uint32_t)(r0 >> 32) ^ k1);
    const uint32_t b3 = (uint32_t)r0;                                   // scalar
    k0 += W0; k1 += W1;
    // third iteration: c3 uniform
    const uint64_t s0 = (uint64_t)M0 * b0;
    const uint64_t s1 = (uint64_t)M1 * b2;
    uint32_t d0 = (uint32_t)(s1 >> 32) ^ b1 ^ k0;
    uint32_t d1 = (uint32_t)s1;
    uint32_t d2 = (uint32_t)(s0 >> 32) ^ (b3 ^ k1);
    uint32_t d3 = (uint32_t)s0;
    k0 += W0; k1 += W1;
#pragma unroll
    for (int r = 3; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)M0 * d0;
        const uint64_t p1 = (uint64_t)M1 * d2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ d1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ d3 ^ k1;
        d1 = (uint32_t)p1;
        d3 = (uint32_t)p0;
        d0 = n0;
        d2 = n2;
        k0 += W0;
        k1 += W1;
    }
    out[0] = d0; out[1] = d1; out[2] = d2; out[3] = d3;
}

__device__ __forceinline__ float word_to_eps(uint32_t word)
{
    return (float)(word >> 8) * 0x1p-24f;      // 24-bit uniform in [0,1), exact
}

// ------------------------------------------------------------------------------------
// element access inside a 16-byte row vector
// ------------------------------------------------------------------------------------
template <int DT> struct Row;
template <> struct Row<NM_DT_F32> {
    static constexpr int VEC = 4;
    static __device__ __forceinline__ float get(const uint4 &v, int c)
    {
        const uint32_t w = c == 0 ? v.x : c == 1 ? v.y : c == 2 ? v.z : v.w;
        return __uint_as_float(w);
    }
};
template <> struct Row<NM_DT_BF16> {
    static constexpr int VEC = 8;
    static __device__ __forceinline__ float get(const uint4 &v, int c)
    {
        const uint32_t w = (c >> 1) == 0 ? v.x : (c >> 1) == 1 ? v.y : (c >> 1) == 2 ? v.z : v.w;
        return __uint_as_float((c & 1) ? (w & 0xffff0000u) : (w << 16));
    }
};

// binary32 -> bf16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t bf16_bits_rne(float f)
{
    const uint32_t b = __float_as_uint(f);
    return (b + 0x7fffu + ((b >> 16) & 1u)) >> 16;
}
// two binary32 -> packed bf16 (lo, hi), round to nearest even: one v_cvt_pk_bf16_f32
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi)
{
    const f32x2_t v = {lo, hi};
    const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    uint32_t u;
    __builtin_memcpy(&u, &b, 4);
    return u;
}

}  // namespace nm
