// approx-MVUE 4:8 prune + compress (appendix, "Additional sparsity results": the approximate 2:4 method of
// Sec. 4.4 carried over to a block of eight).  Four elements are drawn one after the other without replacement, each
// with probability a_j / (sum of the magnitudes not yet drawn); a drawn element is kept with the value a_k / p_k,
// p_k = the probability that k is among the four (eq. (8): what unbiasedness requires).
//
// p_k has no short closed form for four draws; it is computed from its definition, organised by the SET of elements
// drawn so far (the next draw depends on that set only).  With f(U) = probability that the first |U| draws are
// exactly the set U:
//     f({}) = 1,   f(U) = sum_{k in U} g(U \ k) * a_k,   g(V) = f(V) / rest(V),   rest(V) = sum of the magnitudes outside V,
//     p_k = sum over the 4-sets U that contain k of f(U).
// 1 + 8 + 28 + 56 = 93 divisions and about a thousand multiply-adds per block, all in binary32 with one rounding per
// operation and a fixed order (sets in ascending order of their bit mask, elements in ascending position, rest(V) as
// the sum of the low four positions outside V plus the sum of the high four outside V, never by subtraction), so
// that the result is reproducible bit for bit.  This kernel is bound by that arithmetic, not by memory: one thread
// owns one block (8 tokens of one column), and every set index below is a compile-time constant, so f and g live in
// registers.
//
// gfx950's sparse matrix instructions are 4:2 only: this is a prune + storage format, not a GEMM operand.
//     vals[(G*O + o)*8 + 4*b + s]   s-th kept value (ascending position) of octet b = 0, 1 of 16-token group G
//     meta32[G*O + o]               bits [16b + 3s + 2 : 16b + 3s] = position (0..7) of that value
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"
#include "smfmac_common.h"       // static_for
#include "prune_common.h"

namespace nm {

constexpr int popc8(unsigned v) { int c = 0; for (int k = 0; k < 8; ++k) c += (int)((v >> k) & 1u); return c; }
constexpr int top_bit4(unsigned v) { int t = 0; for (int k = 0; k < 4; ++k) if ((v >> k) & 1u) t = k; return t; }

// One draw among eight positions: r[] holds the magnitudes still in the block (0 where already drawn).
// Threshold walk: t = eps * total; the first position whose running sum exceeds t.  When none does (rounding, or
// nothing non-zero left) the last position with a non-zero magnitude, else the lowest position not taken.
__device__ __forceinline__ int draw_of_eight(const float (&r)[8], uint32_t word, uint32_t taken)
{
    float run[8];
    run[0] = r[0];
#pragma unroll
    for (int k = 1; k < 8; ++k) run[k] = run[k - 1] + r[k];
    const float t = word_to_eps(word) * run[7];
    int first = -1;
    uint32_t nzmask = 0;
#pragma unroll
    for (int k = 7; k >= 0; --k) {
        first = (t < run[k]) ? k : first;
        nzmask |= (r[k] > 0.0f ? 1u : 0u) << k;
    }
    if (first >= 0) return first;
    if (nzmask) return 31 - __clz((int)nzmask);
    return __ffs((int)(~taken & 0xffu)) - 1;
}

template <int DT, bool DENSE>
__global__ __launch_bounds__(256) void prune_4of8_approx_kernel(
    const void *__restrict__ g_, int64_t n_octets, int64_t O, int64_t ldg, uint32_t key0, uint32_t key1, uint32_t stream_id,
    void *__restrict__ vals_, uint32_t *__restrict__ meta32, void *__restrict__ dense_, int64_t ldd)
{
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;          // = block index of the random source: octet row * O + o
    if (n >= n_octets * O) return;
    const int64_t oc = n / O, o = n - oc * O;

    float x[8], m[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        if constexpr (DT == NM_DT_F32) x[k] = ((const float *)g_)[(oc * 8 + k) * ldg + o];
        else x[k] = __uint_as_float((uint32_t)((const uint16_t *)g_)[(oc * 8 + k) * ldg + o] << 16);
        m[k] = fabsf(x[k]);
    }

    // four uniforms: one Philox call per block, counter (blk low, blk high, stream, 3)
    uint32_t w4[4];
    philox4x32_10((uint32_t)n, (uint32_t)((uint64_t)n >> 32), stream_id, 3u, key0, key1, w4);

    uint32_t taken = 0;
    {
        float r[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) r[k] = m[k];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int k = draw_of_eight(r, w4[d], taken);
            taken |= 1u << k;
#pragma unroll
            for (int j = 0; j < 8; ++j) r[j] = (j == k) ? 0.0f : r[j];
        }
    }
    int nz = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) nz += m[k] > 0.0f ? 1 : 0;

    float value[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) value[k] = x[k];                         // at most four non-zeros: all kept unchanged
    if (nz > 4) {
        // ascending-position sums of every subset of the low four and of the high four positions (index = member mask)
        float lo[16], hi[16];
        static_for<16>([&](auto s_c) {
            constexpr unsigned S = decltype(s_c)::value;
            if constexpr (S != 0) {
                constexpr int t = top_bit4(S);
                constexpr unsigned rest = S & ~(1u << t);
                if constexpr (rest == 0) { lo[S] = m[t]; hi[S] = m[4 + t]; }
                else { lo[S] = lo[rest] + m[t]; hi[S] = hi[rest] + m[4 + t]; }
            }
        });
        float f[256], gq[256], p[8];
        bool p_started[8] = {false, false, false, false, false, false, false, false};
        static_for<5>([&](auto size_c) {
            constexpr int SIZE = decltype(size_c)::value;
            static_for<256>([&](auto u_c) {
                constexpr unsigned U = decltype(u_c)::value;
                if constexpr (popc8(U) == SIZE) {
                    if constexpr (SIZE == 0) f[U] = 1.0f;
                    else {
                        bool first = true;
                        static_for<8>([&](auto k_c) {
                            constexpr int k = decltype(k_c)::value;
                            if constexpr ((U >> k) & 1u) {
                                const float term = gq[U & ~(1u << k)] * m[k];
                                f[U] = first ? term : f[U] + term;
                                first = false;
                            }
                        });
                    }
                    if constexpr (SIZE < 4) {
                        constexpr unsigned out_lo = ~U & 0xfu, out_hi = (~U >> 4) & 0xfu;      // positions outside U
                        gq[U] = f[U] / (lo[out_lo] + hi[out_hi]);
                    } else {
                        static_for<8>([&](auto k_c) {
                            constexpr int k = decltype(k_c)::value;
                            if constexpr ((U >> k) & 1u) {
                                p[k] = p_started[k] ? p[k] + f[U] : f[U];
                                p_started[k] = true;
                            }
                        });
                    }
                }
            });
        });
        const float total = lo[15] + hi[15];
#pragma unroll
        for (int k = 0; k < 8; ++k) value[k] = copysignf(fminf(m[k] / p[k], total), x[k]);
    }

    // kept values in ascending position; index word of this octet: 3 bits per kept position
    constexpr int ESZ = DT == NM_DT_F32 ? 4 : 2;
    const int64_t G = oc >> 1;
    const int b = (int)(oc & 1);
    float kv[4] = {0.f, 0.f, 0.f, 0.f};
    uint32_t md = 0;
    int s = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const bool kept = (taken >> k) & 1u;
#pragma unroll
        for (int j = 0; j < 4; ++j) kv[j] = (kept && s == j) ? value[k] : kv[j];
        md |= kept ? ((uint32_t)k << (3 * s)) : 0u;
        s += kept ? 1 : 0;
    }
    char *vp = (char *)vals_ + ((G * O + o) * 8 + 4 * b) * ESZ;
    uint32_t st[4];                                   // the values as stored (binary32 words, or bf16 codes)
    if constexpr (DT == NM_DT_F32) {
#pragma unroll
        for (int j = 0; j < 4; ++j) st[j] = __float_as_uint(kv[j]);
        *(uint4 *)vp = make_uint4(st[0], st[1], st[2], st[3]);
    } else {
        const uint32_t w0 = pack_bf16_rne(kv[0], kv[1]), w1 = pack_bf16_rne(kv[2], kv[3]);
        st[0] = w0 & 0xffffu; st[1] = w0 >> 16; st[2] = w1 & 0xffffu; st[3] = w1 >> 16;
        *(uint2 *)vp = make_uint2(w0, w1);
    }
    ((uint16_t *)meta32)[(G * O + o) * 2 + b] = (uint16_t)md;

    if constexpr (DENSE) {
        int sd = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const bool kept = (taken >> k) & 1u;
            uint32_t v = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) v = (kept && sd == j) ? st[j] : v;
            sd += kept ? 1 : 0;
            if constexpr (DT == NM_DT_F32) ((uint32_t *)dense_)[(oc * 8 + k) * ldd + o] = v;
            else ((uint16_t *)dense_)[(oc * 8 + k) * ldd + o] = (uint16_t)v;
        }
    }
}

hipError_t launch_prune_4of8_approx(int dt, const void *g, int64_t T, int64_t O, int64_t ldg, uint64_t seed, uint32_t stream_id,
                                    void *vals, uint32_t *meta32, void *dense, int64_t ldd, hipStream_t st)
{
    const int64_t octets = T / 8, threads = octets * O;
    if (threads == 0) return hipSuccess;
    const int64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffll) return hipErrorInvalidConfiguration;
#define NM_P48(DT, DENSE)                                                                                              \
    hipLaunchKernelGGL((prune_4of8_approx_kernel<DT, DENSE>), dim3((unsigned)blocks), dim3(256), 0, st, g, octets, O, ldg, \
                       (uint32_t)seed, (uint32_t)(seed >> 32), stream_id, vals, meta32, dense, ldd)
    if (dt == NM_DT_F32) { if (dense) NM_P48(NM_DT_F32, true); else NM_P48(NM_DT_F32, false); }
    else { if (dense) NM_P48(NM_DT_BF16, true); else NM_P48(NM_DT_BF16, false); }
#undef NM_P48
    return hipGetLastError();
}

}  // namespace nm
