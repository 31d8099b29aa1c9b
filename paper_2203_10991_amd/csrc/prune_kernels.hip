// Fused MVUE prune + compress kernels for gfx950 (wave64).
//
// One thread owns one 16-token group of VEC columns (VEC = one 16-byte load: 8 bf16 or
// 4 fp32 columns).  Blocks (pairs / quads) run along the token axis, i.e. down the rows of
// the thread's own column, so no cross-lane exchange is needed: 16 coalesced 16-byte row
// loads in, 128 contiguous bytes of kept values + VEC 16-bit index words out.
//
// The decision arithmetic is binary32 with one rounding per operation (compiled with
// -ffp-contract=off) so that masks are reproducible bit for bit from (g, seed, stream).
//
//   MVUE 1:2 ........ Sec. 4.1, eq. (6); threshold sampling as in App. B.1
//   optimal 2:4 ..... Sec. 4.2 (eqs. (8), (12), (14)) and App. A.2 (cases 1-3)
//   approx 2:4 ...... Sec. 4.4 (two magnitude-proportional draws, kept value a/p)
//   8-bit output .... Sec. 5 (FP8 neural gradients on top of 2:4), stochastic rounding for the unbiasedness Sec. 3 asks for
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"
#include "smfmac_common.h"       // static_for
#include "prune_common.h"

namespace nm {

// ------------------------------------------------------------------------------------
// MVUE 1:2 on one pair: returns kept position (0/1) and the kept value (unrounded).
// ------------------------------------------------------------------------------------
__device__ __forceinline__ void select_1of2(float x0, float x1, uint32_t word, uint32_t &kept, float &value)
{
    const float m0 = fabsf(x0), m1 = fabsf(x1);
    const float s = m0 + m1;
    const float t = word_to_eps(word) * s;
    const bool keep0 = (m1 == 0.0f) | (t < m0);       // a zero never wins against a non-zero
    kept = keep0 ? 0u : 1u;
    value = copysignf(s, keep0 ? x0 : x1);
}

// ------------------------------------------------------------------------------------
// optimal MVUE 2:4 on one quad.
// Ranking key, most significant first: magnitude bits, then 3 - position (among equal
// magnitudes the higher position ranks lower), ..., the position itself, the sign.  The last two
// never decide an order (the code above them is unique); they ride along so that the kept
// elements' positions and signs come out of the sorted keys.  bf16 magnitudes leave the low
// 16 bits free, so the key fits 32 bits and is made straight from the packed row word (two
// columns per word): one merge of the column's half with the position constant, one rotate
// that moves the sign from the top to bit 0.  fp32 uses a 64-bit key.
// ------------------------------------------------------------------------------------
template <int DT> struct Key;
template <> struct Key<NM_DT_BF16> {
    typedef uint32_t type;
    // w: row word holding columns (2j, 2j+1); half: which of the two
    static __device__ __forceinline__ type make(const uint4 &v, int c, int pos)
    {
        const uint32_t w = (c >> 1) == 0 ? v.x : (c >> 1) == 1 ? v.y : (c >> 1) == 2 ? v.z : v.w;
        const uint32_t code = ((3u - (uint32_t)pos) << 14) | (uint32_t)pos;          // lands in key bits [16:15] and [2:1]
        const uint32_t d = (c & 1) ? ((w & 0xffff0000u) | code) : ((w << 16) | code);
        return __builtin_rotateleft32(d, 1);              // magnitude [31:17], 3-pos [16:15], pos [2:1], sign [0]
    }
    static __device__ __forceinline__ float mag(type k) { return __uint_as_float((k >> 1) & 0x7fff0000u); }
    static __device__ __forceinline__ uint32_t pos(type k) { return (k >> 1) & 3u; }
    static __device__ __forceinline__ float with_sign(float m, type k) { return __uint_as_float(__float_as_uint(m) | (k << 31)); }
};
template <> struct Key<NM_DT_F32> {
    typedef uint64_t type;
    static __device__ __forceinline__ type make(const uint4 &v, int c, int pos)
    {
        const uint32_t b = c == 0 ? v.x : c == 1 ? v.y : c == 2 ? v.z : v.w;
        return ((uint64_t)(b & 0x7fffffffu) << 8) | ((3u - (uint32_t)pos) << 3) | ((uint32_t)pos << 1) | (b >> 31);
    }
    static __device__ __forceinline__ float mag(type k) { return __uint_as_float((uint32_t)(k >> 8)); }
    static __device__ __forceinline__ uint32_t pos(type k) { return ((uint32_t)k >> 1) & 3u; }
    static __device__ __forceinline__ float with_sign(float m, type k) { return __uint_as_float(__float_as_uint(m) | ((uint32_t)k << 31)); }
};

template <typename K> __device__ __forceinline__ void order2(K &a, K &b)
{
    const K lo = a < b ? a : b;
    const K hi = a < b ? b : a;
    a = lo;
    b = hi;
}
// ascending sort of four distinct keys.  64-bit keys: the 5-comparator network.  32-bit keys: the two middle keys
// come from three-input instructions -- with x <= X and y <= Y the sorted pairs and m = min(X, Y) >= min(x, y), the
// second key is the median and the third the maximum of {x, y, m} -- nine operations instead of ten.
__device__ __forceinline__ void sort4(uint64_t &k1, uint64_t &k2, uint64_t &k3, uint64_t &k4)
{
    order2(k1, k2); order2(k3, k4); order2(k1, k3); order2(k2, k4); order2(k2, k3);
}
__device__ __forceinline__ void sort4(uint32_t &k1, uint32_t &k2, uint32_t &k3, uint32_t &k4)
{
    order2(k1, k2); order2(k3, k4);
    const uint32_t x = k1, X = k2, y = k3, Y = k4;
    const uint32_t m = X < Y ? X : Y;
    k1 = x < y ? x : y;
    k4 = X < Y ? Y : X;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(k2) : "v"(x), "v"(y), "v"(m));
    asm("v_max3_u32 %0, %1, %2, %3" : "=v"(k3) : "v"(x), "v"(y), "v"(m));
}

// out0/out1: kept values in ascending position; nib = pos0 | pos1 << 2.  Straight-line code: the case
// analysis and the walk over the pair probabilities are lane masks and selects, no divergent branch.
template <int DT>
__device__ __forceinline__ void select_2of4(typename Key<DT>::type k1, typename Key<DT>::type k2, typename Key<DT>::type k3,
                                            typename Key<DT>::type k4, uint32_t word, float &out0, float &out1, uint32_t &nib)
{
    typedef Key<DT> KT;
    sort4(k1, k2, k3, k4);
    const float a1 = KT::mag(k1), a2 = KT::mag(k2), a3 = KT::mag(k3), a4 = KT::mag(k4);

    const float s12 = a1 + a2;
    const float s123 = s12 + a3;
    const float s = s123 + a4;
    const float u = fmaf(2.0f, a1, a3);                    // 2*a1 is exact: one rounding, as in (2*a1) + a3
    const bool case1 = a4 <= u;
    const bool case12 = case1 | (a4 <= s123);              // else case 3: a4 dominates

    // cumulative thresholds on t = eps * D.  Cases 1-2: D = 2(a1+a2+a3+a4), walk p13,p14,p23,p24,p34.
    // Case 3: D = a1+a2+a3, partner of a4 is a1 / a2 / a3; expressed in the same chain.
    const float t = word_to_eps(word) * (case12 ? s + s : s123);
    const float c13 = u - a4;                                                   // counts in case 1 only
    const float f4 = case12 ? 4.0f : 1.0f;                                     // (one select for both scaled thresholds: the products are exact)
    const float c14 = f4 * a1;
    const float d34 = s123 - a4;
    const float n23 = case1 ? (fmaf(2.0f, a2, a3) - a4) : (d34 + d34);
    const float c23 = 4.0f * a1 + n23;                                          // counts in cases 1-2 only
    const float c24 = f4 * s12;

    // the first threshold above t decides the pair: 13, 14, 23, 24, else 34 (case 3: 14, 24, else 34)
    const bool lt13 = case1 & (t < c13), lt14 = t < c14, lt23 = case12 & (t < c23), lt24 = t < c24;
    const bool first_is_1 = lt13 | lt14;
    const bool first_is_2 = lt23 | lt24;
    const bool second_is_3 = case12 & (lt13 | (!lt14 & lt23));
    const typename KT::type ka = first_is_1 ? k1 : (first_is_2 ? k2 : k3);
    const typename KT::type kb = second_is_3 ? k3 : k4;

    const float half_s = 0.5f * s;
    const float va = KT::with_sign(case12 ? half_s : s123, ka);                // a_i / p_i
    const float vb = KT::with_sign(case12 ? half_s : a4, kb);
    const uint32_t pa = KT::pos(ka), pb = KT::pos(kb);
    const bool swap = pa > pb;
    out0 = swap ? vb : va;
    out1 = swap ? va : vb;
    nib = swap ? (pb | (pa << 2)) : (pa | (pb << 2));
}

// ------------------------------------------------------------------------------------
// approx-MVUE 2:4 on one quad (Sec. 4.4): one element drawn with probability a_i/sum, a second from
// the other three with probability a_j/(sum - a_i); both kept with value a_k/p_k, p_k the section's
// inclusion probability, i.e.  sum / (1 + sum_{l != k} a_l/(sum - a_l)).  No ranking: position order.
// A draw is a threshold walk over the running sums (t = eps * total, first position whose running
// sum exceeds t); when none does -- rounding, or nothing non-zero left -- it falls on the last
// position with a non-zero magnitude, else on the lowest position not taken, so a zero never beats a
// non-zero and padding falls on the lowest-index zeros.  "sum - a_l" and the sum over l != k are
// formed from the other terms (no cancellation when one element carries the sum).  The six
// divisions are IEEE binary32 divisions.
// ------------------------------------------------------------------------------------
__device__ __forceinline__ void select_2of4_approx(float x0, float x1, float x2, float x3, uint32_t word1, uint32_t word2,
                                                   float &out0, float &out1, uint32_t &nib)
{
    // Straight-line code: draws are lane masks (one per position), everything else selects.
    const float m0 = fabsf(x0), m1 = fabsf(x1), m2 = fabsf(x2), m3 = fabsf(x3);
    const float c1 = m0 + m1, c2 = c1 + m2, total = c2 + m3;
    // first draw.  (t < total would pick position 3, and so does the fallback whenever m3 > 0; with m3 == 0 the
    // total equals c2 and the test cannot hold: one expression covers both.)
    const float t = word_to_eps(word1) * total;
    const bool w0 = t < m0, w1 = t < c1, w2 = t < c2;                           // walk
    const bool n0 = m0 > 0.0f, n1 = m1 > 0.0f, n2 = m2 > 0.0f, n3 = m3 > 0.0f;
    const bool i0 = w0 | (!w1 & !w2 & !n3 & !n2 & !n1);                         // (fallback on position 0: nothing non-zero above it)
    const bool i1 = !w0 & (w1 | (!w2 & !n3 & !n2 & n1));
    const bool i2 = !w0 & !w1 & (w2 | (!n3 & n2));
    const bool i3 = !w0 & !w1 & !w2 & n3;
    // second draw on the block without the first element
    const float r0 = i0 ? 0.0f : m0, r1 = i1 ? 0.0f : m1, r2 = i2 ? 0.0f : m2, r3 = i3 ? 0.0f : m3;
    const float d1 = r0 + r1, d2 = d1 + r2, rest = d2 + r3;
    const float t2 = word_to_eps(word2) * rest;
    const bool u0 = t2 < r0, u1 = t2 < d1, u2 = t2 < d2;
    const bool q0 = r0 > 0.0f, q1 = r1 > 0.0f, q2 = r2 > 0.0f, q3 = r3 > 0.0f;
    const bool none = !q0 & !q1 & !q2 & !q3;                                    // nothing non-zero left: lowest position not taken
    const bool fall = !u0 & !u1 & !u2;
    const bool j0 = u0 | (fall & ((!q3 & !q2 & !q1 & q0) | (none & !i0)));
    const bool j1 = !u0 & (u1 | (!u2 & ((!q3 & !q2 & q1) | (none & i0))));
    const bool j2 = !u0 & !u1 & (u2 | (!q3 & q2));
    const bool j3 = fall & q3;
    // kept values: sum / (1 + sum over the other three of a_l / (sum - a_l)), "sum - a_l" from the other three
    const float s23 = m2 + m3;
    const float o0 = m1 + s23, o1 = m0 + s23, o2 = c1 + m3, o3 = c2;
    const float e0 = m0 / o0, e1 = m1 / o1, e2 = m2 / o2, e3 = m3 / o3;         // (0/0 of a zero element is discarded below)
    const float v0 = n0 ? e0 : 0.0f, v1 = n1 ? e1 : 0.0f, v2 = n2 ? e2 : 0.0f, v3 = n3 ? e3 : 0.0f;
    const float di = 1.0f + ((((i0 ? 0.0f : v0) + (i1 ? 0.0f : v1)) + (i2 ? 0.0f : v2)) + (i3 ? 0.0f : v3));
    const float dj = 1.0f + ((((j0 ? 0.0f : v0) + (j1 ? 0.0f : v1)) + (j2 ? 0.0f : v2)) + (j3 ? 0.0f : v3));
    const float xi = i0 ? x0 : i1 ? x1 : i2 ? x2 : x3;
    const float xj = j0 ? x0 : j1 ? x1 : j2 ? x2 : x3;
    const float vi = copysignf(total / di, xi), vj = copysignf(total / dj, xj);
    const uint32_t pi = i0 ? 0u : i1 ? 1u : i2 ? 2u : 3u, pj = j0 ? 0u : j1 ? 1u : j2 ? 2u : 3u;
    const bool swap = pi > pj;
    out0 = swap ? vj : vi;
    out1 = swap ? vi : vj;
    nib = swap ? (pj | (pi << 2)) : (pi | (pj << 2));
}

// ------------------------------------------------------------------------------------
// MVUE 1:4 on one quad (appendix, additional sparsity results: MVUE 1:2 on a block of four): position k is kept
// with probability a_k/sum and emits sign(x_k) * sum.  Same threshold walk and fallback as the draws above.
// Stored in the 2:4 container: the quad's other slot is a +0 at the lowest other position.
// ------------------------------------------------------------------------------------
__device__ __forceinline__ void select_1of4(float x0, float x1, float x2, float x3, uint32_t word,
                                            float &out0, float &out1, uint32_t &nib)
{
    const float m0 = fabsf(x0), m1 = fabsf(x1), m2 = fabsf(x2), m3 = fabsf(x3);
    const float c1 = m0 + m1, c2 = c1 + m2, total = c2 + m3;
    const float t = word_to_eps(word) * total;
    const bool w0 = t < m0, w1 = t < c1, w2 = t < c2;
    const bool n1 = m1 > 0.0f, n2 = m2 > 0.0f, n3 = m3 > 0.0f;
    const bool i0 = w0 | (!w1 & !w2 & !n3 & !n2 & !n1);
    const bool i1 = !w0 & (w1 | (!w2 & !n3 & !n2 & n1));
    const bool i2 = !w0 & !w1 & (w2 | (!n3 & n2));
    const float xi = i0 ? x0 : i1 ? x1 : i2 ? x2 : x3;
    const float v = copysignf(total, xi);
    const uint32_t k = i0 ? 0u : i1 ? 1u : i2 ? 2u : 3u;
    out0 = i0 ? v : 0.0f;
    out1 = i0 ? 0.0f : v;
    nib = i0 ? 4u : (k << 2);                  // (0, 1) when position 0 is kept, else (0, k)
}

// ------------------------------------------------------------------------------------
// Greedy N:M (the comparison method of the paper's tables, Sec. 4.1 ablation and Sec. 5: keep the n largest
// magnitudes of the block, values unchanged).  Deterministic: no random words.  Among equal magnitudes the lower
// position is kept -- the order of the ranking keys above.
// ------------------------------------------------------------------------------------
__device__ __forceinline__ void select_greedy_1of2(float x0, float x1, uint32_t &kept, float &value)
{
    const bool keep1 = fabsf(x1) > fabsf(x0);
    kept = keep1 ? 1u : 0u;
    value = keep1 ? x1 : x0;
}
template <int DT>
__device__ __forceinline__ void select_greedy_2of4(typename Key<DT>::type k1, typename Key<DT>::type k2, typename Key<DT>::type k3,
                                                   typename Key<DT>::type k4, float &out0, float &out1, uint32_t &nib)
{
    typedef Key<DT> KT;
    sort4(k1, k2, k3, k4);
    const float va = KT::with_sign(KT::mag(k3), k3), vb = KT::with_sign(KT::mag(k4), k4);
    const uint32_t pa = KT::pos(k3), pb = KT::pos(k4);
    const bool swap = pa > pb;
    out0 = swap ? vb : va;
    out1 = swap ? va : vb;
    nib = swap ? (pb | (pa << 2)) : (pa | (pb << 2));
}

// ------------------------------------------------------------------------------------
// the fused kernel
// ------------------------------------------------------------------------------------
// M = 2: MVUE 1:2; M = 4: EST = 0 the optimal MVUE 2:4, 1 approx-MVUE 2:4, 2 MVUE 1:4; EST = 4 (either M): Greedy;
// DENSE: also write theta(g)
// PROD: the kernel is also the PRODUCER of the neural gradient (eq. (2): g_l = Diag(f'(z_l)) W^T g_{l+1}): g_ holds
// u = W^T g_{l+1} (the dense backward GEMM's output) and dense_ / ldd the derivative factor d = f'(z_l); each row of
// g_l = u * d (one binary32 product per element, rounded to the storage type) is formed in registers, written once to
// gout_ -- the next layer's backward GEMM needs it dense -- and pruned from there: g_l is never read back.
struct ProdArg { const void *d; int64_t ldd; void *gout; int64_t ldgo; };

template <int DT>
__device__ __forceinline__ uint4 producer_row(const uint4 &u, const uint4 &d)
{
    uint4 r;
    if constexpr (DT == NM_DT_F32) {
        r.x = __float_as_uint(__uint_as_float(u.x) * __uint_as_float(d.x)); r.y = __float_as_uint(__uint_as_float(u.y) * __uint_as_float(d.y));
        r.z = __float_as_uint(__uint_as_float(u.z) * __uint_as_float(d.z)); r.w = __float_as_uint(__uint_as_float(u.w) * __uint_as_float(d.w));
    } else {
        auto mul2 = [](uint32_t a, uint32_t b) {
            return pack_bf16_rne(__uint_as_float(a << 16) * __uint_as_float(b << 16),
                                 __uint_as_float(a & 0xffff0000u) * __uint_as_float(b & 0xffff0000u));
        };
        r.x = mul2(u.x, d.x); r.y = mul2(u.y, d.y); r.z = mul2(u.z, d.z); r.w = mul2(u.w, d.w);
    }
    return r;
}

// HI0: the caller guarantees that every Philox call index of the launch is below 2^32 (the launcher checks the
// tensor's size): counter words 1-3 are then wave-uniform and the generator's first rounds run partly on the scalar unit.
// Streaming (non-temporal) forms of a 16-byte load and store
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
// (the pointers are to global memory; said explicitly, because an address that went through an opaque asm statement
// would otherwise be loaded from with the generic form, which counts as an LDS operation too)
#define NM_GLOBAL __attribute__((address_space(1)))
__device__ __forceinline__ uint4 load_stream(const void *p)
{
    const u32x4_t t = __builtin_nontemporal_load((const NM_GLOBAL u32x4_t *)p);
    return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ uint4 load_global(const void *p)
{
    const u32x4_t t = *(const NM_GLOBAL u32x4_t *)p;
    return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void store_stream(void *p, const uint4 &v)
{
    const u32x4_t t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, (u32x4_t *)p);
}

template <int DT, int M, int EST, bool DENSE, bool PROD = false, bool HI0 = false, bool NT = false>
__device__ __forceinline__ void prune_compress_body(
    const void *__restrict__ g_, int64_t n_groups, int64_t O, int64_t ldg,
    uint32_t key0, uint32_t key1, uint32_t stream_id,
    void *__restrict__ vals_, uint16_t *__restrict__ meta_, void *__restrict__ dense_, int64_t ldd, ProdArg pa = ProdArg{})
{
    static_assert(!(PROD && DENSE), "the producer form writes g_l, not theta(g_l)");
    constexpr int VEC = Row<DT>::VEC;
    constexpr int ESZ = DT == NM_DT_F32 ? 4 : 2;
    const int64_t ncg = O / VEC;
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= n_groups * ncg) return;                 // (NT: the launcher has checked that the thread count is a multiple of 64: whole waves leave)
    const int64_t G = n / ncg;
    const int64_t col0 = (n - G * ncg) * VEC;

    const char *gp = (const char *)g_ + ((G * 16) * ldg + col0) * ESZ;
    // The second half of the rows is requested only after the first block row is decided (an opaque copy of the
    // address keeps those loads from being hoisted): their latency hides under the arithmetic of the rows already
    // here, and fewer registers are live at once, so one more wave fits each SIMD.
    uint4 rows[16];
    const char *dp_in = nullptr;
    char *gop = nullptr;
    if constexpr (PROD) {
        dp_in = (const char *)pa.d + ((G * 16) * pa.ldd + col0) * ESZ;
        gop = (char *)pa.gout + ((G * 16) * pa.ldgo + col0) * ESZ;
    }
    auto fetch_rows = [&](const char *base, const char *dbase, int first) {
#pragma unroll
        for (int r = first; r < first + 8; ++r) {
            if constexpr (NT) rows[r] = load_stream(base + (int64_t)r * ldg * ESZ);
            else rows[r] = load_global(base + (int64_t)r * ldg * ESZ);
            if constexpr (PROD) {
                if constexpr (NT) {
                    rows[r] = producer_row<DT>(rows[r], load_stream(dbase + (int64_t)r * pa.ldd * ESZ));
                    store_stream(gop + (int64_t)r * pa.ldgo * ESZ, rows[r]);
                } else {
                    rows[r] = producer_row<DT>(rows[r], load_global(dbase + (int64_t)r * pa.ldd * ESZ));
                    *(uint4 *)(gop + (int64_t)r * pa.ldgo * ESZ) = rows[r];
                }
            }
        }
    };
    fetch_rows(gp, dp_in, 0);

    // kept values per column in the slot order of the group format, as stored: binary32 words, or bf16 pairs
    // (slots 2i, 2i+1) packed as soon as a block row is decided, which keeps the live registers low
    constexpr int KW = DT == NM_DT_F32 ? 8 : 4;      // words per column
    uint32_t kept[VEC][KW];
    uint32_t md[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) md[c] = 0;
    auto put2 = [&](int c, int i, float v0, float v1) {      // slots 2i and 2i+1 of column c
        if constexpr (DT == NM_DT_F32) { kept[c][2 * i] = __float_as_uint(v0); kept[c][2 * i + 1] = __float_as_uint(v1); }
        else kept[c][i] = pack_bf16_rne(v0, v1);
    };

    constexpr int BLOCK_ROWS = 16 / M;       // pair rows (8) or quad rows (4) in the group
    float held[VEC];                         // 1:2: the kept value of the even pair row, until its partner is known
    // one uniform per block: four blocks share a Philox call (counter blk/4, last counter word 0);
    // approx-MVUE draws twice: two blocks share a call (counter blk/2, last counter word 1)
    constexpr int WPB = EST == 1 ? 2 : 1;            // words per block
    constexpr int CTR_SHIFT = EST == 1 ? 1 : 2;
    constexpr uint32_t DOMAIN = EST == 1 ? 1u : 0u;
    [[maybe_unused]] const uint32_t ctr0 = (uint32_t)(((uint64_t)(G * BLOCK_ROWS) * (uint64_t)O + (uint64_t)col0) >> CTR_SHIFT);   // call index of block row 0
#pragma unroll
    for (int b = 0; b < BLOCK_ROWS; ++b) {
        if (b == 1) {
            const char *gp2 = gp, *dp2 = dp_in;
            asm volatile("" : "+v"(gp2));               // an address the compiler cannot see through
            fetch_rows(gp2, dp2, 8);
        }
        const uint64_t blk0 = (uint64_t)(G * BLOCK_ROWS + b) * (uint64_t)O + (uint64_t)col0;
        uint32_t words[VEC * WPB];
        if constexpr (EST != 4) {
#pragma unroll
            for (int q = 0; q < VEC * WPB / 4; ++q) {
                const uint64_t ctr = (blk0 >> CTR_SHIFT) + q;
                uint32_t w4[4];
                // HI0: the call index fits 32 bits, and block row b adds b * O (a multiple of 8) to the block index
                if constexpr (HI0) philox4x32_10_uniform_c123(ctr0 + (uint32_t)b * (uint32_t)(O >> CTR_SHIFT) + (uint32_t)q, 0u, stream_id, DOMAIN, key0, key1, w4);
                else philox4x32_10((uint32_t)ctr, (uint32_t)(ctr >> 32), stream_id, DOMAIN, key0, key1, w4);
#pragma unroll
                for (int j = 0; j < 4; ++j) words[4 * q + j] = w4[j];
            }
        }
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            if (M == 2) {
                uint32_t k; float v;
                if constexpr (EST == 4) select_greedy_1of2(Row<DT>::get(rows[2 * b], c), Row<DT>::get(rows[2 * b + 1], c), k, v);
                else
                select_1of2(Row<DT>::get(rows[2 * b], c), Row<DT>::get(rows[2 * b + 1], c), words[c], k, v);
                if (b & 1) put2(c, b >> 1, held[c], v); else held[c] = v;
                md[c] |= ((uint32_t)((b & 1) << 1) | k) << (2 * b);
            } else {
                float v0, v1; uint32_t nib;
                if constexpr (EST == 1)
                    select_2of4_approx(Row<DT>::get(rows[4 * b], c), Row<DT>::get(rows[4 * b + 1], c),
                                       Row<DT>::get(rows[4 * b + 2], c), Row<DT>::get(rows[4 * b + 3], c),
                                       words[2 * c], words[2 * c + 1], v0, v1, nib);
                else if constexpr (EST == 2)
                    select_1of4(Row<DT>::get(rows[4 * b], c), Row<DT>::get(rows[4 * b + 1], c),
                                Row<DT>::get(rows[4 * b + 2], c), Row<DT>::get(rows[4 * b + 3], c), words[c], v0, v1, nib);
                else if constexpr (EST == 4)
                    select_greedy_2of4<DT>(Key<DT>::make(rows[4 * b], c, 0), Key<DT>::make(rows[4 * b + 1], c, 1),
                                           Key<DT>::make(rows[4 * b + 2], c, 2), Key<DT>::make(rows[4 * b + 3], c, 3), v0, v1, nib);
                else
                    select_2of4<DT>(Key<DT>::make(rows[4 * b], c, 0), Key<DT>::make(rows[4 * b + 1], c, 1),
                                    Key<DT>::make(rows[4 * b + 2], c, 2), Key<DT>::make(rows[4 * b + 3], c, 3),
                                    words[c], v0, v1, nib);
                put2(c, b, v0, v1);
                md[c] |= nib << (4 * b);
                __builtin_amdgcn_sched_barrier(0);       // one block at a time: interleaving blocks only lengthens live ranges
            }
        }
    }

    // ---- kept values: 8 per column, VEC columns contiguous = 128 bytes per thread
    char *vp = (char *)vals_ + ((G * O + col0) * 8) * ESZ;            // = vals_ + 128 n: a wave's 64 threads own 8 KB in a row
    [[maybe_unused]] uint16_t *mp_late = nullptr;
    // Streaming stores want whole lines per instruction: the wave's 8 KB go through its own 8 KB of LDS, written as
    // each thread holds them (eight 16-byte pieces at a stride of 128 bytes; piece c of lane l at slot 8l + (c ^ l%8),
    // which spreads the lanes over the banks) and read back so that store k covers bytes [1024 k, 1024 k + 1024).
    // Every lane of the wave is here (the launcher sends only launches made of whole waves to the streaming kernels), and
    // a wave's LDS operations execute in order, so the reads below see the writes above without a workgroup barrier.
    if constexpr (NT) {
        __shared__ __attribute__((aligned(1024))) char xs[4 * 8192];
        uint32_t tid = threadIdx.x;
        asm volatile("" : "+v"(tid) : "v"(kept[VEC - 1][KW - 1]));       // (the addresses below are formed here, after the last block, not carried through the kernel)
        const uint32_t lane = tid & 63u, wave_lds = (tid >> 6) * 8192;
        const int64_t n_late = (int64_t)blockIdx.x * 256 + tid;          // = n
        // byte address of piece p of this lane: 128 lane + 16 (p ^ lane%8) = (128 lane + 16 (lane%8)) ^ 16 p
        const uint32_t wr = wave_lds + lane * 128 + (lane & 7) * 16;
#pragma unroll
        for (int c = 0; c < VEC; ++c)
#pragma unroll
            for (int j = 0; j < KW / 4; ++j) {
                const int piece = c * (KW / 4) + j;
                *(uint4 *)(xs + (wr ^ (uint32_t)(piece * 16))) = make_uint4(kept[c][4 * j], kept[c][4 * j + 1], kept[c][4 * j + 2], kept[c][4 * j + 3]);
            }
        __builtin_amdgcn_wave_barrier();
        // store k, lane l: piece l%8 of the wave's thread 8k + l/8, which sits at slot 8 (8k + l/8) + (l%8 ^ l/8)
        char *wave_base = (char *)vals_ + (n_late - lane) * 128;
        mp_late = meta_ + n_late * VEC;                                   // (G O + col0 = n VEC)
        const uint32_t rd = wave_lds + (8 * (lane >> 3) + ((lane & 7) ^ (lane >> 3))) * 16;
#pragma unroll
        for (int k = 0; k < 8; ++k) store_stream(wave_base + (1024 * k + 16 * lane), *(const uint4 *)(xs + rd + 1024 * k));
    } else {
#pragma unroll
    for (int c = 0; c < VEC; ++c)
#pragma unroll
        for (int j = 0; j < KW / 4; ++j)
            ((uint4 *)vp)[c * (KW / 4) + j] = make_uint4(kept[c][4 * j], kept[c][4 * j + 1], kept[c][4 * j + 2], kept[c][4 * j + 3]);
    }
    // ---- index words
    uint16_t *mp = NT ? mp_late : meta_ + (G * O + col0);
    if (VEC == 8) {
        uint4 o;
        o.x = md[0] | (md[1] << 16); o.y = md[2] | (md[3] << 16);
        o.z = md[4 % VEC] | (md[5 % VEC] << 16); o.w = md[6 % VEC] | (md[7 % VEC] << 16);
        if constexpr (NT) store_stream(mp, o);
        else *(uint4 *)mp = o;
    } else {
        uint2 o;
        o.x = md[0] | (md[1] << 16); o.y = md[2] | (md[3] << 16);
        if constexpr (NT) {
            typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
            const u32x2_t t = {o.x, o.y};
            __builtin_nontemporal_store(t, (u32x2_t *)mp);
        } else *(uint2 *)mp = o;
    }

    // ---- optional dense theta(g)
    if constexpr (DENSE) {
        char *dp = (char *)dense_ + ((G * 16) * ldd + col0) * ESZ;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int q = r >> 2, p = r & 3;             // quad and position inside it
            uint32_t w[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                const uint32_t nib = (md[c] >> (4 * q)) & 0xfu;
                // the stored words of slots 2q and 2q+1 (bf16: the two halves of one word)
                const uint32_t s0 = DT == NM_DT_F32 ? kept[c][(2 * q) % KW] : (kept[c][q % KW] & 0xffffu);
                const uint32_t s1 = DT == NM_DT_F32 ? kept[c][(2 * q + 1) % KW] : (kept[c][q % KW] >> 16);
                w[c] = (nib & 3u) == (uint32_t)p ? s0 : (nib >> 2) == (uint32_t)p ? s1 : 0u;
            }
            uint4 o;
            if (DT == NM_DT_F32) { o.x = w[0]; o.y = w[1]; o.z = w[2]; o.w = w[3]; }
            else {
                o.x = w[0] | (w[1] << 16); o.y = w[2] | (w[3] << 16);
                o.z = w[4 % VEC] | (w[5 % VEC] << 16); o.w = w[6 % VEC] | (w[7 % VEC] << 16);
            }
            *(uint4 *)(dp + (int64_t)r * ldd * ESZ) = o;
        }
    }
}

template <int DT, int M, int EST, bool DENSE>
__global__ __launch_bounds__(256) void prune_compress_kernel(
    const void *__restrict__ g, int64_t n_groups, int64_t O, int64_t ldg, uint32_t key0, uint32_t key1, uint32_t stream_id,
    void *__restrict__ vals, uint16_t *__restrict__ meta, void *__restrict__ dense, int64_t ldd)
{
    prune_compress_body<DT, M, EST, DENSE>(g, n_groups, O, ldg, key0, key1, stream_id, vals, meta, dense, ldd);
}
// The streaming form (no dense output): its 32 KB of LDS let five workgroups onto a CU, so five waves per SIMD is
// what the registers are budgeted for (four for the instances that need more than 96).
// HI0: every Philox call index of the launch is below 2^32, which the launcher has checked.
template <int DT, int M, int EST, bool HI0>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu((DT == NM_DT_BF16 && (EST == 1 || (M == 2 && EST == 0))) ? 4 : 5, 5))) void prune_compress_stream_kernel(
    const void *__restrict__ g, int64_t n_groups, int64_t O, int64_t ldg, uint32_t key0, uint32_t key1, uint32_t stream_id,
    void *__restrict__ vals, uint16_t *__restrict__ meta)
{
    prune_compress_body<DT, M, EST, false, false, HI0, true>(g, n_groups, O, ldg, key0, key1, stream_id, vals, meta, nullptr, 0);
}
template <int DT, int M, int EST, bool NT>
__global__ __launch_bounds__(256) void prune_producer_kernel(
    const void *__restrict__ u, int64_t n_groups, int64_t O, int64_t ldu, uint32_t key0, uint32_t key1, uint32_t stream_id,
    void *__restrict__ vals, uint16_t *__restrict__ meta, ProdArg pa)
{
    prune_compress_body<DT, M, EST, false, true, false, NT>(u, n_groups, O, ldu, key0, key1, stream_id, vals, meta, nullptr, 0, pa);
}
// The bf16 optimal-2:4 kernel without the dense output needs 98 registers as the compiler would have it, two more
// than let a fifth wave onto each SIMD; asked for five waves it fits 96 without spilling.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(5, 5))) void prune_compress_bf16_2of4_kernel(
    const void *__restrict__ g, int64_t n_groups, int64_t O, int64_t ldg, uint32_t key0, uint32_t key1, uint32_t stream_id,
    void *__restrict__ vals, uint16_t *__restrict__ meta)
{
    prune_compress_body<NM_DT_BF16, 4, 0, false, false, true>(g, n_groups, O, ldg, key0, key1, stream_id, vals, meta, nullptr, 0);
}
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(5, 5))) void prune_compress_bf16_2of4_stream_kernel(
    const void *__restrict__ g, int64_t n_groups, int64_t O, int64_t ldg, uint32_t key0, uint32_t key1, uint32_t stream_id,
    void *__restrict__ vals, uint16_t *__restrict__ meta)
{
    prune_compress_body<NM_DT_BF16, 4, 0, false, false, true, true>(g, n_groups, O, ldg, key0, key1, stream_id, vals, meta, nullptr, 0);
}

// ------------------------------------------------------------------------------------
// 2:4 prune with 8-bit output (Sec. 5, 8-bit rows: FP8 neural gradients; Sec. 3: the quantiser of a neural
// gradient has to be unbiased).  Selection and kept values as above, in binary32; each kept value is multiplied
// by `scale` and rounded stochastically to e5m2 with 16 random bits: with lo <= |x| < hi neighbours on the e5m2
// grid and f = (|x| - lo)/(hi - lo), the result is hi iff r16 + floor(f * 2^16) >= 2^16.
//   |x| >= 57344 (the largest finite e5m2) saturates; a NaN gives an e5m2 NaN.
// Rounding words: one Philox call per four blocks with last counter word 2, word blk%4; its low half rounds the
// first kept value, its high half the second.
// Output: 32-token groups, vals8[(G*O + o)*16 + 2i + s], meta32[G*O + o] (nibble i = quad i).
// ------------------------------------------------------------------------------------
// The rounding itself is one instruction: v_cvt_sr_bf8_f32 adds the top 21 bits of its random operand to the 21
// mantissa bits it discards (subnormal results: to the bits below the 2^-16 step) and truncates, which with the 16
// rounding bits in the operand's top half and zeros below them is exactly the rule above -- checked against the
// integer formulation for every rounding word over a million inputs of every exponent.  It overflows to infinity
// where this format saturates, so the value is clamped to +-57344 first; the code lands in byte BYTE of `word`.
template <int BYTE>
__device__ __forceinline__ uint32_t sr_e5m2_into(uint32_t word, float x, uint32_t r_top)
{
    const float c = __builtin_amdgcn_fmed3f(x, -57344.0f, 57344.0f);
    return (uint32_t)__builtin_amdgcn_cvt_sr_bf8_f32(c, (int)r_top, (int)word, BYTE);
}

// HI0: every Philox call index of the launch is below 2^32 (checked by the launcher), see prune_compress_body
template <int DT, int EST, bool HI0>
__global__ __launch_bounds__(256) void prune_compress_q8_kernel(
    const void *__restrict__ g_, int64_t n_groups, int64_t O, int64_t ldg, uint32_t key0, uint32_t key1, uint32_t stream_id,
    float scale, const float *__restrict__ scale_dev, uint8_t *__restrict__ vals8, uint32_t *__restrict__ meta32)
{
    if (scale_dev) scale = scale_dev[0];            // the scale as a device value (element 0 of a scale record)
    auto philox = [&](uint64_t ctr, uint32_t domain, uint32_t (&w4)[4]) {
        if constexpr (HI0) philox4x32_10_uniform_c123((uint32_t)ctr, 0u, stream_id, domain, key0, key1, w4);
        else philox4x32_10((uint32_t)ctr, (uint32_t)(ctr >> 32), stream_id, domain, key0, key1, w4);
    };
    constexpr int VEC = Row<DT>::VEC;
    constexpr int ESZ = DT == NM_DT_F32 ? 4 : 2;
    const int64_t ncg = O / VEC;
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= n_groups * ncg) return;
    const int64_t G = n / ncg;
    const int64_t col0 = (n - G * ncg) * VEC;
    const char *gp = (const char *)g_ + ((G * 32) * ldg + col0) * ESZ;

    // rows live in two halves of 8 (two quad rows each); a half is refilled with the rows 16 further down as soon
    // as its quads are decided, through an address the compiler cannot see through (keeps the loads where they are)
    uint4 rows[16];
#pragma unroll
    for (int r = 0; r < 8; ++r) rows[r] = load_global(gp + (int64_t)r * ldg * ESZ);

    uint32_t kept[VEC][4];        // 16 e5m2 codes per column
    uint32_t md[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) { md[c] = 0; kept[c][0] = kept[c][1] = kept[c][2] = kept[c][3] = 0; }

    static_for<8>([&](auto b_c) {                       // quad row b: tensor rows 4b .. 4b+3, held in rows[(4b) % 16 ..]
        constexpr int b = decltype(b_c)::value;
        if constexpr (b == 1 || b == 2 || b == 4) {
            const int first = b == 1 ? 8 : b == 2 ? 16 : 24;
            const char *gp2 = gp;
            asm volatile("" : "+v"(gp2));
#pragma unroll
            for (int r = 0; r < 8; ++r) rows[(first + r) % 16] = load_global(gp2 + (int64_t)(first + r) * ldg * ESZ);
        }
        constexpr int R0 = (4 * b) % 16;
        if constexpr (EST == 3) {
            // MVUE 1:2: the quad row holds two pair rows; the kept value of pair row 2b+pr is slot pr of quad b, rounded
            // with the low half of the pair block's rounding word
            static_for<2>([&](auto pr_c) {
                constexpr int pr = decltype(pr_c)::value;
                const uint64_t pblk0 = (uint64_t)(G * 16 + 2 * b + pr) * (uint64_t)O + (uint64_t)col0;
                uint32_t sel[VEC], rnd1[VEC];
#pragma unroll
                for (int q = 0; q < VEC / 4; ++q) {
                    const uint64_t ctr = (pblk0 >> 2) + q;
                    uint32_t w4[4];
                    philox(ctr, 0u, w4);
#pragma unroll
                    for (int j = 0; j < 4; ++j) sel[4 * q + j] = w4[j];
                    philox(ctr, 2u, w4);
#pragma unroll
                    for (int j = 0; j < 4; ++j) rnd1[4 * q + j] = w4[j];
                }
#pragma unroll
                for (int c = 0; c < VEC; ++c) {
                    uint32_t k; float v;
                    select_1of2(Row<DT>::get(rows[R0 + 2 * pr], c), Row<DT>::get(rows[R0 + 2 * pr + 1], c), sel[c], k, v);
                    kept[c][b / 2] = sr_e5m2_into<2 * (b & 1) + pr>(kept[c][b / 2], v * scale, rnd1[c] << 16);
                    md[c] |= ((uint32_t)(pr << 1) | k) << (4 * b + 2 * pr);
                }
                __builtin_amdgcn_sched_barrier(0);
            });
            return;
        }
        const uint64_t blk0 = (uint64_t)(G * 8 + b) * (uint64_t)O + (uint64_t)col0;
        constexpr int WPB = EST == 1 ? 2 : 1;
        uint32_t words[VEC * WPB], rnd[VEC];
#pragma unroll
        for (int q = 0; q < VEC * WPB / 4; ++q) {
            const uint64_t ctr = (blk0 >> (EST == 1 ? 1 : 2)) + q;
            uint32_t w4[4];
            philox(ctr, EST == 1 ? 1u : 0u, w4);
#pragma unroll
            for (int j = 0; j < 4; ++j) words[4 * q + j] = w4[j];
        }
#pragma unroll
        for (int q = 0; q < VEC / 4; ++q) {
            const uint64_t ctr = (blk0 >> 2) + q;
            uint32_t w4[4];
            philox(ctr, 2u, w4);
#pragma unroll
            for (int j = 0; j < 4; ++j) rnd[4 * q + j] = w4[j];
        }
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            float v0, v1; uint32_t nib;
            if constexpr (EST == 1)
                select_2of4_approx(Row<DT>::get(rows[R0], c), Row<DT>::get(rows[R0 + 1], c),
                                   Row<DT>::get(rows[R0 + 2], c), Row<DT>::get(rows[R0 + 3], c),
                                   words[2 * c], words[2 * c + 1], v0, v1, nib);
            else
                select_2of4<DT>(Key<DT>::make(rows[R0], c, 0), Key<DT>::make(rows[R0 + 1], c, 1),
                                Key<DT>::make(rows[R0 + 2], c, 2), Key<DT>::make(rows[R0 + 3], c, 3),
                                words[c], v0, v1, nib);
            kept[c][b / 2] = sr_e5m2_into<2 * (b & 1)>(kept[c][b / 2], v0 * scale, rnd[c] << 16);
            kept[c][b / 2] = sr_e5m2_into<2 * (b & 1) + 1>(kept[c][b / 2], v1 * scale, rnd[c] & 0xffff0000u);
            md[c] |= nib << (4 * b);
            __builtin_amdgcn_sched_barrier(0);
        }
    });

    // 16 bytes per column, VEC columns contiguous; one index word per column
    uint4 *vp = (uint4 *)(vals8 + (G * O + col0) * 16);
#pragma unroll
    for (int c = 0; c < VEC; ++c) vp[c] = make_uint4(kept[c][0], kept[c][1], kept[c][2], kept[c][3]);
    uint4 *mp = (uint4 *)(meta32 + (G * O + col0));
#pragma unroll
    for (int c = 0; c < VEC / 4; ++c) mp[c] = make_uint4(md[4 * c], md[4 * c + 1], md[4 * c + 2], md[4 * c + 3]);
}

template <int DT, int EST>
static hipError_t launch_prune_q8_t(const void *g, int64_t T, int64_t O, int64_t ldg, uint64_t seed, uint32_t stream_id,
                                    float scale, const float *scale_dev, uint8_t *vals8, uint32_t *meta32, hipStream_t st)
{
    const int64_t groups = T / 32, threads = groups * (O / Row<DT>::VEC);
    if (threads == 0) return hipSuccess;
    if ((threads + 255) / 256 > 0x7fffffffll) return hipErrorInvalidConfiguration;
    // The bf16 optimal-2:4 kernel has a form for launches whose call indices (at most T*O/16 + 1) all lie below 2^32 (2^35 elements is a safe bound);
    // the other instances run the general code, which the larger tensors take too.
    if constexpr (DT == NM_DT_BF16 && EST == 0) {
        if ((uint64_t)T * (uint64_t)O <= ((uint64_t)1 << 35)) {
            hipLaunchKernelGGL((prune_compress_q8_kernel<DT, EST, true>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                               g, groups, O, ldg, (uint32_t)seed, (uint32_t)(seed >> 32), stream_id, scale, scale_dev, vals8, meta32);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((prune_compress_q8_kernel<DT, EST, false>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                       g, groups, O, ldg, (uint32_t)seed, (uint32_t)(seed >> 32), stream_id, scale, scale_dev, vals8, meta32);
    return hipGetLastError();
}

hipError_t launch_prune_q8(int dt, int est, const void *g, int64_t T, int64_t O, int64_t ldg, uint64_t seed,
                           uint32_t stream_id, float scale, const float *scale_dev, uint8_t *vals8, uint32_t *meta32, hipStream_t st)
{
#define NM_PRUNE8(DT, EST) launch_prune_q8_t<DT, EST>(g, T, O, ldg, seed, stream_id, scale, scale_dev, vals8, meta32, st)
    // est: 0 optimal MVUE 2:4, 1 approx-MVUE 2:4, 3 MVUE 1:2
    if (dt == NM_DT_F32) return est == 3 ? NM_PRUNE8(NM_DT_F32, 3) : est == 1 ? NM_PRUNE8(NM_DT_F32, 1) : NM_PRUNE8(NM_DT_F32, 0);
    return est == 3 ? NM_PRUNE8(NM_DT_BF16, 3) : est == 1 ? NM_PRUNE8(NM_DT_BF16, 1) : NM_PRUNE8(NM_DT_BF16, 0);
#undef NM_PRUNE8
}

// ------------------------------------------------------------------------------------
// MVUE 2:4 (or 1:2) prune + compress of a gradient stored TRANSPOSED: gT is [O x T], tokens contiguous, so a quad
// (a pair) is four (two) adjacent elements of a row.  Same estimators, same random stream and block index (blk = (t/4)*O + o) as the
// kernels above: the output equals theirs on the transposed tensor, bit for bit.
// Workgroup = 16 columns o x 16 token groups; a thread owns one (o, group): it loads the group's 16 tokens as one
// contiguous piece (16 threads of a column read 512 or 1024 consecutive bytes), decides its four quads, and the
// kept values and index words go through LDS so that the stores run along o (16 x 16 or 32 bytes contiguous per
// token group), which is how the group format is laid out.
// ------------------------------------------------------------------------------------
template <int DT, int EST>
__global__ __launch_bounds__(256) void prune_compress_t_kernel(
    const void *__restrict__ gT_, int64_t n_groups, int64_t O, int64_t ldt, uint32_t key0, uint32_t key1, uint32_t stream_id,
    void *__restrict__ vals_, uint16_t *__restrict__ meta_)
{
    constexpr int ESZ = DT == NM_DT_F32 ? 4 : 2;
    constexpr int VW = 16 * ESZ / 4;                       // 32-bit words of a group's 16 tokens: 8 (bf16) or 16 (fp32)
    constexpr int KW = 8 * ESZ / 4;                        // words of its 8 kept values: 4 or 8
    __shared__ uint32_t kept_s[16][16][KW + 1];            // [group][column][word] (+1: no bank conflicts on the way in)
    __shared__ uint16_t meta_s[16][16];
    const int tid = threadIdx.x, oi = tid >> 4, gi = tid & 15;
    // consecutive workgroups walk along the tokens of the same 16 columns
    const int64_t gblocks = (n_groups + 15) / 16;
    const int64_t ob = (int64_t)blockIdx.x / gblocks, gb = (int64_t)blockIdx.x % gblocks;
    const int64_t o = ob * 16 + oi, G = gb * 16 + gi;
    const bool live = o < O && G < n_groups;

    uint32_t w[VW];
#pragma unroll
    for (int j = 0; j < VW; ++j) w[j] = 0;
    if (live) {
        const uint4 *src = (const uint4 *)((const char *)gT_ + (o * ldt + G * 16) * ESZ);
#pragma unroll
        for (int j = 0; j < VW / 4; ++j) { const uint4 v = src[j]; w[4 * j] = v.x; w[4 * j + 1] = v.y; w[4 * j + 2] = v.z; w[4 * j + 3] = v.w; }
    }
    auto elem_bits = [&](int t) -> uint32_t {             // token t of the group as binary32 bits
        if constexpr (DT == NM_DT_F32) return w[t];
        else return (t & 1) ? (w[t >> 1] & 0xffff0000u) : (w[t >> 1] << 16);
    };
    // Random words.  A wave holds 4 columns (a multiple of 4 onwards) x 16 groups, and the blocks of those 4 columns
    // in one quad row share their Philox calls (one call for the optimal estimator, two for approx-MVUE), as in the
    // token-major kernels.  Lane (a, gi) makes the calls of quad row a of group gi for the wave's columns and leaves
    // the words in LDS; lane (j, gi) then picks, for each quad row, the words of its own column j.
    constexpr int WPC = EST == 1 ? 8 : 4;                  // words per (group, block row) of a wave's four columns
    constexpr int RB = EST == 3 ? 8 : 4;                   // block rows of a group: 8 pair rows (1:2) or 4 quad rows
    __shared__ __attribute__((aligned(16))) uint32_t rnd_s[4][RB][16][WPC];      // [wave][block row][group][word]
    {
        const int wave = tid >> 6, a = oi & 3;
#pragma unroll
        for (int rb = 0; rb < RB / 4; ++rb) {
            const int b = a + 4 * rb;
            const uint64_t blk0 = (uint64_t)(G * RB + b) * (uint64_t)O + (uint64_t)(o - a);
#pragma unroll
            for (int c = 0; c < WPC / 4; ++c) {
                uint32_t r4[4];
                const uint64_t ctr = (blk0 >> (EST == 1 ? 1 : 2)) + c;
                philox4x32_10((uint32_t)ctr, (uint32_t)(ctr >> 32), stream_id, EST == 1 ? 1u : 0u, key0, key1, r4);
                *(uint4 *)&rnd_s[wave][b][gi][4 * c] = make_uint4(r4[0], r4[1], r4[2], r4[3]);
            }
        }
    }
    __syncthreads();
    uint32_t md = 0;
    uint32_t kept[KW];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float v0, v1; uint32_t nib;
        if constexpr (EST == 3) {
            // two pairs fill the two slots of quad i: the first keeps position 0 or 1, the second 2 or 3
            uint32_t k0, k1;
            select_1of2(__uint_as_float(elem_bits(4 * i)), __uint_as_float(elem_bits(4 * i + 1)),
                        rnd_s[tid >> 6][2 * i][gi][oi & 3], k0, v0);
            select_1of2(__uint_as_float(elem_bits(4 * i + 2)), __uint_as_float(elem_bits(4 * i + 3)),
                        rnd_s[tid >> 6][2 * i + 1][gi][oi & 3], k1, v1);
            nib = k0 | ((2u | k1) << 2);
        } else {
        const uint32_t *rw = rnd_s[tid >> 6][i][gi];
        if constexpr (EST == 1) {
            const uint2 wab = *(const uint2 *)&rw[2 * (oi & 3)];
            select_2of4_approx(__uint_as_float(elem_bits(4 * i)), __uint_as_float(elem_bits(4 * i + 1)),
                               __uint_as_float(elem_bits(4 * i + 2)), __uint_as_float(elem_bits(4 * i + 3)), wab.x, wab.y, v0, v1, nib);
        } else {
            const uint32_t word = rw[oi & 3];
            // (the ranking keys are built from one-element "rows": the element sits where column 0 of a row would)
            uint4 e[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t b = elem_bits(4 * i + p);
                e[p] = make_uint4(DT == NM_DT_F32 ? b : (b >> 16), 0u, 0u, 0u);
            }
            select_2of4<DT>(Key<DT>::make(e[0], 0, 0), Key<DT>::make(e[1], 0, 1), Key<DT>::make(e[2], 0, 2), Key<DT>::make(e[3], 0, 3),
                            word, v0, v1, nib);
        }
        }
        if constexpr (DT == NM_DT_F32) { kept[2 * i] = __float_as_uint(v0); kept[2 * i + 1] = __float_as_uint(v1); }
        else kept[i] = pack_bf16_rne(v0, v1);
        md |= nib << (4 * i);
    }
#pragma unroll
    for (int j = 0; j < KW; ++j) kept_s[gi][oi][j] = kept[j];
    meta_s[gi][oi] = (uint16_t)md;
    __syncthreads();
    // second half: thread (group gj, column oj) stores what thread (oj, gj) computed: 16 threads write one token group's run along o
    const int gj = tid >> 4, oj = tid & 15;
    const int64_t o2 = ob * 16 + oj, G2 = gb * 16 + gj;
    if (o2 < O && G2 < n_groups) {
        uint32_t *dst = (uint32_t *)((char *)vals_ + ((G2 * O + o2) * 8) * ESZ);
        // streaming stores (16 threads write whole lines; measured 1.5 % faster than plain ones; streaming LOADS of the
        // 32- or 64-byte pieces a thread reads measured no faster)
        store_stream(dst, make_uint4(kept_s[gj][oj][0], kept_s[gj][oj][1], kept_s[gj][oj][2], kept_s[gj][oj][3]));
        if constexpr (KW == 8) store_stream(dst + 4, make_uint4(kept_s[gj][oj][4], kept_s[gj][oj][5], kept_s[gj][oj][6], kept_s[gj][oj][7]));
        meta_[G2 * O + o2] = meta_s[gj][oj];
    }
}

template <int DT, int EST>
static hipError_t launch_prune_t_t(const void *gT, int64_t T, int64_t O, int64_t ldt, uint64_t seed, uint32_t stream_id,
                                   void *vals, uint16_t *meta, hipStream_t st)
{
    const int64_t groups = T / 16;
    if (groups == 0 || O == 0) return hipSuccess;
    const int64_t blocks = ((groups + 15) / 16) * ((O + 15) / 16);
    if (blocks > 0x7fffffffll) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((prune_compress_t_kernel<DT, EST>), dim3((unsigned)blocks), dim3(256), 0, st, gT, groups, O, ldt, (uint32_t)seed,
                       (uint32_t)(seed >> 32), stream_id, vals, meta);
    return hipGetLastError();
}

hipError_t launch_prune_transposed(int dt, int est, const void *gT, int64_t T, int64_t O, int64_t ldt, uint64_t seed,
                                   uint32_t stream_id, void *vals, uint16_t *meta, hipStream_t st)
{
    // est: 0 optimal MVUE 2:4, 1 approx-MVUE 2:4, 3 MVUE 1:2
#define NM_T_CASE(DT_, EST_) \
    if (dt == DT_ && est == EST_) return launch_prune_t_t<DT_, EST_>(gT, T, O, ldt, seed, stream_id, vals, meta, st)
    NM_T_CASE(NM_DT_F32, 0); NM_T_CASE(NM_DT_F32, 1); NM_T_CASE(NM_DT_F32, 3);
    NM_T_CASE(NM_DT_BF16, 0); NM_T_CASE(NM_DT_BF16, 1); NM_T_CASE(NM_DT_BF16, 3);
#undef NM_T_CASE
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------------------------
// The 8-bit prune of a gradient stored TRANSPOSED (gT [O x T], tokens contiguous): selection, kept values, scaling and
// stochastic rounding as in prune_compress_q8_kernel, with the same random streams and block indices, so the output
// equals that kernel's on the transposed tensor bit for bit.  Same workgroup shape as prune_compress_t_kernel with
// 32-token groups: a thread owns one (column, group), loads the group's 32 tokens as one contiguous piece (64 or 128
// bytes), decides its eight quads (sixteen pairs), and the 16 codes and the index word go through LDS so that the
// stores run along o.
// ------------------------------------------------------------------------------------
template <int DT, int EST>
__global__ __launch_bounds__(256) void prune_compress_q8_t_kernel(
    const void *__restrict__ gT_, int64_t n_groups, int64_t O, int64_t ldt, uint32_t key0, uint32_t key1, uint32_t stream_id,
    float scale, const float *__restrict__ scale_dev, uint8_t *__restrict__ vals8, uint32_t *__restrict__ meta32)
{
    if (scale_dev) scale = scale_dev[0];
    constexpr int ESZ = DT == NM_DT_F32 ? 4 : 2;
    constexpr int VW = 32 * ESZ / 4;                       // 32-bit words of a group's 32 tokens: 16 (bf16) or 32 (fp32)
    __shared__ uint32_t kept_s[16][16][5];                 // [group][column][word] (+1: no bank conflicts on the way in)
    __shared__ uint32_t meta_s[16][16];
    const int tid = threadIdx.x, oi = tid >> 4, gi = tid & 15;
    const int64_t gblocks = (n_groups + 15) / 16;          // consecutive workgroups walk along the tokens of the same 16 columns
    const int64_t ob = (int64_t)blockIdx.x / gblocks, gb = (int64_t)blockIdx.x % gblocks;
    const int64_t o = ob * 16 + oi, G = gb * 16 + gi;
    const bool live = o < O && G < n_groups;

    uint32_t w[VW];
#pragma unroll
    for (int j = 0; j < VW; ++j) w[j] = 0;
    if (live) {
        const uint4 *src = (const uint4 *)((const char *)gT_ + (o * ldt + G * 32) * ESZ);
#pragma unroll
        for (int j = 0; j < VW / 4; ++j) { const uint4 v = src[j]; w[4 * j] = v.x; w[4 * j + 1] = v.y; w[4 * j + 2] = v.z; w[4 * j + 3] = v.w; }
    }
    auto elem_bits = [&](int t) -> uint32_t {             // token t of the group as binary32 bits
        if constexpr (DT == NM_DT_F32) return w[t];
        else return (t & 1) ? (w[t >> 1] & 0xffff0000u) : (w[t >> 1] << 16);
    };
    // Random words, shared as in prune_compress_t_kernel: a wave holds 4 columns x 16 groups; lane (a, gi) makes the
    // calls of block rows a, a + 4, ... of group gi for the wave's four columns -- the selection words (last counter
    // word 0, or 1 with two calls for approx-MVUE) and the rounding words (last counter word 2) -- and leaves them in LDS.
    constexpr int RB = EST == 3 ? 16 : 8;                  // block rows of a group: 16 pair rows (1:2) or 8 quad rows
    constexpr int SELW = EST == 1 ? 8 : 4;                 // selection words per block row of four columns
    constexpr int WPC = SELW + 4;                          // + their four rounding words
    __shared__ __attribute__((aligned(16))) uint32_t rnd_s[4][RB][16][WPC];      // [wave][block row][group][word]
    {
        const int wave = tid >> 6, a = oi & 3;
#pragma unroll
        for (int rb = 0; rb < RB / 4; ++rb) {
            const int b = a + 4 * rb;
            const uint64_t blk0 = (uint64_t)(G * RB + b) * (uint64_t)O + (uint64_t)(o - a);
            uint32_t r4[4];
#pragma unroll
            for (int c = 0; c < SELW / 4; ++c) {
                const uint64_t ctr = (blk0 >> (EST == 1 ? 1 : 2)) + c;
                philox4x32_10((uint32_t)ctr, (uint32_t)(ctr >> 32), stream_id, EST == 1 ? 1u : 0u, key0, key1, r4);
                *(uint4 *)&rnd_s[wave][b][gi][4 * c] = make_uint4(r4[0], r4[1], r4[2], r4[3]);
            }
            const uint64_t ctr = blk0 >> 2;
            philox4x32_10((uint32_t)ctr, (uint32_t)(ctr >> 32), stream_id, 2u, key0, key1, r4);
            *(uint4 *)&rnd_s[wave][b][gi][SELW] = make_uint4(r4[0], r4[1], r4[2], r4[3]);
        }
    }
    __syncthreads();
    uint32_t md = 0;
    uint32_t kept[4] = {0u, 0u, 0u, 0u};
    const int col = oi & 3;
    static_for<8>([&](auto i_c) {                           // quad i of the group: tokens 4i .. 4i+3, codes 2i and 2i+1
        constexpr int i = decltype(i_c)::value;
        float v0, v1; uint32_t nib, r0, r1;                 // r0, r1: rounding bits of the two kept values, in the top half
        if constexpr (EST == 3) {
            const uint32_t *ra = rnd_s[tid >> 6][2 * i][gi], *rb = rnd_s[tid >> 6][2 * i + 1][gi];
            uint32_t k0, k1;
            select_1of2(__uint_as_float(elem_bits(4 * i)), __uint_as_float(elem_bits(4 * i + 1)), ra[col], k0, v0);
            select_1of2(__uint_as_float(elem_bits(4 * i + 2)), __uint_as_float(elem_bits(4 * i + 3)), rb[col], k1, v1);
            nib = k0 | ((2u | k1) << 2);
            r0 = ra[SELW + col] << 16;                      // each pair block rounds with the low half of its own word
            r1 = rb[SELW + col] << 16;
        } else {
            const uint32_t *rw = rnd_s[tid >> 6][i][gi];
            if constexpr (EST == 1) {
                const uint2 wab = *(const uint2 *)&rw[2 * col];
                select_2of4_approx(__uint_as_float(elem_bits(4 * i)), __uint_as_float(elem_bits(4 * i + 1)),
                                   __uint_as_float(elem_bits(4 * i + 2)), __uint_as_float(elem_bits(4 * i + 3)), wab.x, wab.y, v0, v1, nib);
            } else {
                uint4 e[4];                                 // one-element "rows": the element sits where column 0 of a row would
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const uint32_t b = elem_bits(4 * i + p);
                    e[p] = make_uint4(DT == NM_DT_F32 ? b : (b >> 16), 0u, 0u, 0u);
                }
                select_2of4<DT>(Key<DT>::make(e[0], 0, 0), Key<DT>::make(e[1], 0, 1), Key<DT>::make(e[2], 0, 2), Key<DT>::make(e[3], 0, 3),
                                rw[col], v0, v1, nib);
            }
            const uint32_t r = rw[SELW + col];
            r0 = r << 16;
            r1 = r & 0xffff0000u;
        }
        kept[i / 2] = sr_e5m2_into<2 * (i & 1)>(kept[i / 2], v0 * scale, r0);
        kept[i / 2] = sr_e5m2_into<2 * (i & 1) + 1>(kept[i / 2], v1 * scale, r1);
        md |= nib << (4 * i);
    });
#pragma unroll
    for (int j = 0; j < 4; ++j) kept_s[gi][oi][j] = kept[j];
    meta_s[gi][oi] = md;
    __syncthreads();
    // second half: thread (group gj, column oj) stores what thread (oj, gj) computed: 16 threads write one token group's run along o
    const int gj = tid >> 4, oj = tid & 15;
    const int64_t o2 = ob * 16 + oj, G2 = gb * 16 + gj;
    if (o2 < O && G2 < n_groups) {
        *(uint4 *)(vals8 + (G2 * O + o2) * 16) = make_uint4(kept_s[gj][oj][0], kept_s[gj][oj][1], kept_s[gj][oj][2], kept_s[gj][oj][3]);
        meta32[G2 * O + o2] = meta_s[gj][oj];
    }
}

template <int DT, int EST>
static hipError_t launch_prune_q8_t_t(const void *gT, int64_t T, int64_t O, int64_t ldt, uint64_t seed, uint32_t stream_id, float scale,
                                      const float *scale_dev, uint8_t *vals8, uint32_t *meta32, hipStream_t st)
{
    const int64_t groups = T / 32;
    if (groups == 0 || O == 0) return hipSuccess;
    const int64_t blocks = ((groups + 15) / 16) * ((O + 15) / 16);
    if (blocks > 0x7fffffffll) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((prune_compress_q8_t_kernel<DT, EST>), dim3((unsigned)blocks), dim3(256), 0, st, gT, groups, O, ldt, (uint32_t)seed,
                       (uint32_t)(seed >> 32), stream_id, scale, scale_dev, vals8, meta32);
    return hipGetLastError();
}

hipError_t launch_prune_q8_transposed(int dt, int est, const void *gT, int64_t T, int64_t O, int64_t ldt, uint64_t seed,
                                      uint32_t stream_id, float scale, const float *scale_dev, uint8_t *vals8, uint32_t *meta32,
                                      hipStream_t st)
{
    // est: 0 optimal MVUE 2:4, 1 approx-MVUE 2:4, 3 MVUE 1:2
#define NM_T8_CASE(DT_, EST_) \
    if (dt == DT_ && est == EST_) return launch_prune_q8_t_t<DT_, EST_>(gT, T, O, ldt, seed, stream_id, scale, scale_dev, vals8, meta32, st)
    NM_T8_CASE(NM_DT_F32, 0); NM_T8_CASE(NM_DT_F32, 1); NM_T8_CASE(NM_DT_F32, 3);
    NM_T8_CASE(NM_DT_BF16, 0); NM_T8_CASE(NM_DT_BF16, 1); NM_T8_CASE(NM_DT_BF16, 3);
#undef NM_T8_CASE
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------------------------
// nm_compress: dense n:m tensor -> group format.  Same thread tiling as above.
// ------------------------------------------------------------------------------------
// The per-wave transpose of prune_compress_body as a function: every lane of the wave hands in the eight 16-byte pieces
// it would have stored at vals + 128 n (n = its thread number in the launch); the wave stores them as eight streaming
// stores of 1 KB of whole lines each.  xs: the workgroup's 32 KB of LDS.  Whole waves only.
__device__ __forceinline__ void store_wave_pieces_stream(void *vals_, char *xs, const uint4 (&piece)[8])
{
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave_lds = (tid >> 6) * 8192;
    const uint32_t wr = wave_lds + lane * 128 + (lane & 7) * 16;         // piece p at slot 8 lane + (p ^ lane % 8)
#pragma unroll
    for (int p = 0; p < 8; ++p) *(uint4 *)(xs + (wr ^ (uint32_t)(p * 16))) = piece[p];
    __builtin_amdgcn_wave_barrier();
    const int64_t n = (int64_t)blockIdx.x * 256 + tid;
    char *wave_base = (char *)vals_ + (n - lane) * 128;
    const uint32_t rd = wave_lds + (8 * (lane >> 3) + ((lane & 7) ^ (lane >> 3))) * 16;
#pragma unroll
    for (int k = 0; k < 8; ++k) store_stream(wave_base + (1024 * k + 16 * lane), *(const uint4 *)(xs + rd + 1024 * k));
}

template <int DT, int M, bool NT = false>
__global__ __launch_bounds__(256) void compress_kernel(
    const void *__restrict__ d_, int64_t n_groups, int64_t O, int64_t ld,
    void *__restrict__ vals_, uint16_t *__restrict__ meta_, int32_t *__restrict__ bad)
{
    constexpr int VEC = Row<DT>::VEC;
    constexpr int ESZ = DT == NM_DT_F32 ? 4 : 2;
    const int64_t ncg = O / VEC;
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= n_groups * ncg) return;
    const int64_t G = n / ncg;
    const int64_t col0 = (n - G * ncg) * VEC;
    const char *gp = (const char *)d_ + ((G * 16) * ld + col0) * ESZ;
    uint4 rows[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) rows[r] = NT ? load_stream(gp + (int64_t)r * ld * ESZ) : load_global(gp + (int64_t)r * ld * ESZ);

    constexpr int KW = DT == NM_DT_F32 ? 8 : 4;      // stored words per column: binary32 values, or bf16 pairs packed at once
    uint32_t kept[VEC][KW];
    uint32_t md[VEC];
    int nbad = 0;
#pragma unroll
    for (int c = 0; c < VEC; ++c) md[c] = 0;
    // quad row by quad row (the rows of a finished one are dead), one quad at a time
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            float x[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) x[p] = Row<DT>::get(rows[4 * i + p], c);
            uint32_t p0, p1;
            if (M == 4) {
                const uint32_t nz = (x[0] != 0.0f ? 1u : 0u) | (x[1] != 0.0f ? 2u : 0u) |
                                    (x[2] != 0.0f ? 4u : 0u) | (x[3] != 0.0f ? 8u : 0u);
                // straight-line: fewer than two non-zeros are padded with the lowest zero positions (one if one is
                // missing, two if both are)
                uint32_t taken = nz;
                const int cnt = __popc(nz);
                nbad += cnt > 2 ? 1 : 0;
                const uint32_t z1 = ~taken & 0xfu;
                taken |= cnt < 2 ? (z1 & (0u - z1)) : 0u;                  // lowest zero
                const uint32_t z2 = ~taken & 0xfu;
                taken |= cnt < 1 ? (z2 & (0u - z2)) : 0u;
                p0 = (uint32_t)__ffs((int)taken) - 1u;
                taken &= taken - 1u;
                p1 = (uint32_t)__ffs((int)taken) - 1u;
            } else {
                const bool n0 = x[0] != 0.0f, n1 = x[1] != 0.0f, n2 = x[2] != 0.0f, n3 = x[3] != 0.0f;
                nbad += (n0 & n1) + (n2 & n3);
                p0 = (n1 & !n0) ? 1u : 0u;
                p1 = (n3 & !n2) ? 3u : 2u;
            }
            // (two levels of selects on the position's bits: written as a chain of comparisons the compiler made branches of it)
            const uint32_t u0 = __float_as_uint(x[0]), u1 = __float_as_uint(x[1]), u2 = __float_as_uint(x[2]), u3 = __float_as_uint(x[3]);
            const uint32_t k0 = (p0 & 2u) ? ((p0 & 1u) ? u3 : u2) : ((p0 & 1u) ? u1 : u0);
            const uint32_t k1 = (p1 & 2u) ? ((p1 & 1u) ? u3 : u2) : ((p1 & 1u) ? u1 : u0);
            if constexpr (DT == NM_DT_F32) { kept[c][2 * i] = k0; kept[c][2 * i + 1] = k1; }
            else kept[c][i] = (k0 >> 16) | (k1 & 0xffff0000u);        // values are bf16 already: the upper half is exact
            md[c] |= (p0 | (p1 << 2)) << (4 * i);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    char *vp = (char *)vals_ + ((G * O + col0) * 8) * ESZ;            // = vals_ + 128 n
    uint4 piece[8];                                                   // the thread's 128 bytes of vals
#pragma unroll
    for (int c = 0; c < VEC; ++c)
#pragma unroll
        for (int j = 0; j < KW / 4; ++j)
            piece[c * (KW / 4) + j] = make_uint4(kept[c][4 * j], kept[c][4 * j + 1], kept[c][4 * j + 2], kept[c][4 * j + 3]);
    if constexpr (NT) {
        __shared__ __attribute__((aligned(1024))) char xs[4 * 8192];
        store_wave_pieces_stream(vals_, xs, piece);
    } else {
#pragma unroll
        for (int p = 0; p < 8; ++p) ((uint4 *)vp)[p] = piece[p];
    }
    uint16_t *mp = meta_ + (G * O + col0);
    if (VEC == 8) {
        uint4 o;
        o.x = md[0] | (md[1] << 16); o.y = md[2] | (md[3] << 16);
        o.z = md[4 % VEC] | (md[5 % VEC] << 16); o.w = md[6 % VEC] | (md[7 % VEC] << 16);
        *(uint4 *)mp = o;
    } else {
        uint2 o;
        o.x = md[0] | (md[1] << 16); o.y = md[2] | (md[3] << 16);
        *(uint2 *)mp = o;
    }
    if (bad && nbad) atomicAdd(bad, nbad);
}

// ------------------------------------------------------------------------------------
// launchers (called from the C ABI after validation)
// ------------------------------------------------------------------------------------
template <int DT, int M, int EST>
static hipError_t launch_prune_t(const void *g, int64_t T, int64_t O, int64_t ldg, uint64_t seed, uint32_t stream_id,
                                 void *vals, uint16_t *meta, void *dense, int64_t ldd, hipStream_t st)
{
    const int64_t groups = T / 16, threads = groups * (O / Row<DT>::VEC);
    if (threads == 0) return hipSuccess;
    const int64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffll) return hipErrorInvalidConfiguration;
    // The streaming kernels store through whole waves: they take the launches whose thread count is a multiple of 64.
    // hi0: every call index (block / 4, or block / 2 for approx-MVUE's two words per block) lies below 2^32
    const bool hi0 = EST != 4 && (uint64_t)(T / M) * (uint64_t)O <= ((uint64_t)1 << (EST == 1 ? 33 : 34));
    const dim3 grid((unsigned)blocks);
#define NM_ARGS g, groups, O, ldg, (uint32_t)seed, (uint32_t)(seed >> 32), stream_id, vals, meta
    if (dense)
        hipLaunchKernelGGL((prune_compress_kernel<DT, M, EST, true>), grid, dim3(256), 0, st, NM_ARGS, dense, ldd);
    else if (DT == NM_DT_BF16 && M == 4 && EST == 0 && hi0 && threads % 64 == 0)
        hipLaunchKernelGGL(prune_compress_bf16_2of4_stream_kernel, grid, dim3(256), 0, st, NM_ARGS);
    else if (DT == NM_DT_BF16 && M == 4 && EST == 0 && hi0)
        hipLaunchKernelGGL(prune_compress_bf16_2of4_kernel, grid, dim3(256), 0, st, NM_ARGS);
    else if (threads % 64 == 0) {
        if (hi0) hipLaunchKernelGGL((prune_compress_stream_kernel<DT, M, EST, true>), grid, dim3(256), 0, st, NM_ARGS);
        else hipLaunchKernelGGL((prune_compress_stream_kernel<DT, M, EST, false>), grid, dim3(256), 0, st, NM_ARGS);
    } else
        hipLaunchKernelGGL((prune_compress_kernel<DT, M, EST, false>), grid, dim3(256), 0, st, NM_ARGS, dense, ldd);
#undef NM_ARGS
    return hipGetLastError();
}

// g_l = u * d written to gout, and its prune + compress, in one pass.  m = 2: MVUE 1:2; m = 4: est 0 optimal / 1 approx-MVUE 2:4
hipError_t launch_prune_producer(int dt, int m, int est, const void *u, int64_t ldu, const void *d, int64_t ldd, int64_t T, int64_t O,
                                 uint64_t seed, uint32_t stream_id, void *gout, int64_t ldgo, void *vals, uint16_t *meta, hipStream_t st)
{
    const int64_t groups = T / 16, threads = groups * (O / (dt == NM_DT_F32 ? 4 : 8));
    if (threads == 0) return hipSuccess;
    const int64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffll) return hipErrorInvalidConfiguration;
    const ProdArg pa{d, ldd, gout, ldgo};
    // whole waves only on the streaming form (its stores go through the whole wave)
#define NM_PROD(DT, M, EST)                                                                                             \
    do {                                                                                                                \
        if (threads % 64 == 0)                                                                                          \
            hipLaunchKernelGGL((prune_producer_kernel<DT, M, EST, true>), dim3((unsigned)blocks), dim3(256), 0, st, u, groups, O, ldu,  \
                               (uint32_t)seed, (uint32_t)(seed >> 32), stream_id, vals, meta, pa);                      \
        else                                                                                                            \
            hipLaunchKernelGGL((prune_producer_kernel<DT, M, EST, false>), dim3((unsigned)blocks), dim3(256), 0, st, u, groups, O, ldu, \
                               (uint32_t)seed, (uint32_t)(seed >> 32), stream_id, vals, meta, pa);                      \
    } while (0)
    if (dt == NM_DT_F32) { if (m == 2) NM_PROD(NM_DT_F32, 2, 0); else if (est == 1) NM_PROD(NM_DT_F32, 4, 1); else NM_PROD(NM_DT_F32, 4, 0); }
    else { if (m == 2) NM_PROD(NM_DT_BF16, 2, 0); else if (est == 1) NM_PROD(NM_DT_BF16, 4, 1); else NM_PROD(NM_DT_BF16, 4, 0); }
#undef NM_PROD
    return hipGetLastError();
}

// m = 2: est = 0 MVUE 1:2, 4 Greedy 1:2;  m = 4: est = 0 optimal MVUE 2:4, 1 approx-MVUE 2:4, 2 MVUE 1:4, 4 Greedy 2:4
hipError_t launch_prune(int dt, int m, int est, const void *g, int64_t T, int64_t O, int64_t ldg, uint64_t seed,
                        uint32_t stream_id, void *vals, uint16_t *meta, void *dense, int64_t ldd, hipStream_t st)
{
#define NM_PRUNE(DT, M, EST) launch_prune_t<DT, M, EST>(g, T, O, ldg, seed, stream_id, vals, meta, dense, ldd, st)
    if (dt == NM_DT_F32) {
        if (m == 2) return est == 4 ? NM_PRUNE(NM_DT_F32, 2, 4) : NM_PRUNE(NM_DT_F32, 2, 0);
        return est == 1 ? NM_PRUNE(NM_DT_F32, 4, 1) : est == 2 ? NM_PRUNE(NM_DT_F32, 4, 2) : est == 4 ? NM_PRUNE(NM_DT_F32, 4, 4) : NM_PRUNE(NM_DT_F32, 4, 0);
    }
    if (m == 2) return est == 4 ? NM_PRUNE(NM_DT_BF16, 2, 4) : NM_PRUNE(NM_DT_BF16, 2, 0);
    return est == 1 ? NM_PRUNE(NM_DT_BF16, 4, 1) : est == 2 ? NM_PRUNE(NM_DT_BF16, 4, 2) : est == 4 ? NM_PRUNE(NM_DT_BF16, 4, 4) : NM_PRUNE(NM_DT_BF16, 4, 0);
#undef NM_PRUNE
}

template <int DT, int M>
static hipError_t launch_compress_t(const void *d, int64_t T, int64_t O, int64_t ld, void *vals, uint16_t *meta,
                                    int32_t *bad, hipStream_t st)
{
    const int64_t groups = T / 16, threads = groups * (O / Row<DT>::VEC);
    if (threads == 0) return hipSuccess;
    if ((threads + 255) / 256 > 0x7fffffffll) return hipErrorInvalidConfiguration;
    if (threads % 64 == 0)          // whole waves: streaming loads, stores of whole lines through the per-wave transpose
        hipLaunchKernelGGL((compress_kernel<DT, M, true>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                           d, groups, O, ld, vals, meta, bad);
    else
        hipLaunchKernelGGL((compress_kernel<DT, M, false>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                           d, groups, O, ld, vals, meta, bad);
    return hipGetLastError();
}

hipError_t launch_compress(int dt, int m, const void *d, int64_t T, int64_t O, int64_t ld, void *vals,
                           uint16_t *meta, int32_t *bad, hipStream_t st)
{
    if (dt == NM_DT_F32)
        return m == 2 ? launch_compress_t<NM_DT_F32, 2>(d, T, O, ld, vals, meta, bad, st)
                      : launch_compress_t<NM_DT_F32, 4>(d, T, O, ld, vals, meta, bad, st);
    return m == 2 ? launch_compress_t<NM_DT_BF16, 2>(d, T, O, ld, vals, meta, bad, st)
                  : launch_compress_t<NM_DT_BF16, 4>(d, T, O, ld, vals, meta, bad, st);
}

}  // namespace nm
