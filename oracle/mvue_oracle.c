/*
 * mvue_oracle.c -- CPU ORACLE.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, host-only statement of what the MVUE N:M prune -> compress ->
 * update-GEMM path computes, written from the paper (arXiv 2203.10991).  It shares
 * no code with the HIP library and must never be linked, imported or called by
 * the product path: only the tests, the smoke check and the benchmark's
 * cpu_baseline leg use it.
 *
 *   - MVUE 1:2 estimator ............ Sec. 4.1, eq. (6) ("our_method_main"); sampling by a
 *                                      uniform threshold: App. B.1, "Part 1".
 *   - optimal MVUE 2:4 .............. Sec. 4.2 (optimality conditions, eqs. (12),(14)) and
 *                                      App. A.2 (pair probabilities p_ij, cases 1-3).
 *   - approx-MVUE 2:4 ............... Sec. 4.4: two draws without replacement, each proportional
 *                                      to magnitude; kept value a_i/p_i with the inclusion
 *                                      probability p_i of that section.
 *   - MVUE 1:4 ...................... appendix ("Additional sparsity results"): eq. (6) on a block of
 *                                      four, stored in the 2:4 container.
 *   - Greedy N:M .................... the comparison method of the paper's tables (keep the n largest,
 *                                      unchanged): deterministic, biased.
 *   - approx-MVUE 4:8 ............... appendix ("Additional sparsity results"): four magnitude-proportional
 *                                      draws out of eight, kept value a_k/p_k with the exact inclusion
 *                                      probability of the four draws.
 *   - update GEMM ................... eq. (3):  dC/dW_l = g_l h_{l-1}^T; for a convolution (App. B.1, part 1)
 *                                      also without the im2col matrix.
 *   - random source ................. the paper only asks for eps ~ U[0,1) per block; this build
 *                                      fixes Philox4x32-10 (Salmon et al., SC'11) as a pure
 *                                      function of (seed, stream, block index).
 *   - 8-bit neural gradients ........ Sec. 5 (sparsity in all phases + 8-bit quantisation: FP8 neural
 *                                      gradients) with the unbiasedness requirement of Sec. 3:
 *                                      stochastic rounding of the kept values to e5m2.
 *   - compressed format ............. not in the paper (the abstract only counts a halved footprint);
 *                                      defined below.
 *
 * Decision arithmetic is IEEE binary32 with one rounding per written operation
 * (compile with -ffp-contract=off, no fast-math): the paper measures in FP32
 * (Table 2 caption) and the device takes the same decisions in the same
 * precision.  The GEMM is the plain definition in binary64.
 *
 * Compressed N:M operand ("group format").  Tokens (rows of g, the GEMM reduction
 * axis) are cut into groups of 16 = 4 quads.  For group G and column o
 *     vals[(G*O + o)*8 + 2*i + s]   s-th kept value (ascending position) of quad i, i=0..3
 *     meta[ G*O + o ]  (uint16)     bits [4i+1:4i] = position of kept 0, bits [4i+3:4i+2] = kept 1
 * with position in 0..3 inside the quad and kept0 < kept1.  A 1:2 tensor is stored
 * the same way: quad i holds pairs 2i and 2i+1, so kept0 in {0,1}, kept1 in {2,3}.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py (published
 * Philox known answers, closed-form probabilities/variances, exhaustive enumeration of
 * all 2^24 thresholds, brute-force minimum variance, library GEMM; the 8-bit path by a library's
 * float8 decoder and nearest cast, exact rational counts over all 2^16 rounding words, library GEMM;
 * the convolution's update GEMM by a library's convolution weight gradient).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { DT_F32 = 0, DT_BF16 = 1 };

/* ------------------------------------------------------------------------- */
/* storage types                                                              */
/* ------------------------------------------------------------------------- */
static float bits_to_float(uint32_t b) { float f; memcpy(&f, &b, 4); return f; }
static uint32_t float_to_bits(float f) { uint32_t b; memcpy(&b, &f, 4); return b; }

/* bf16 -> binary32 is exact: bf16 is the upper half of a binary32. */
static float bf16_widen(uint16_t h) { return bits_to_float((uint32_t)h << 16); }

/* binary32 -> bf16, round to nearest, ties to even (finite inputs; NaN kept quiet). */
static uint16_t bf16_round(float f)
{
    uint32_t b = float_to_bits(f);
    if ((b & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((b >> 16) | 0x0040u);
    uint32_t lower = b & 0xffffu, upper = b >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) upper += 1u;
    return (uint16_t)upper;
}

static float load_elem(const void *p, int dt, int64_t idx)
{
    return dt == DT_F32 ? ((const float *)p)[idx] : bf16_widen(((const uint16_t *)p)[idx]);
}
/* Store with the storage type's rounding; returns the value as stored. */
static float store_elem(void *p, int dt, int64_t idx, float v)
{
    if (dt == DT_F32) { ((float *)p)[idx] = v; return v; }
    uint16_t h = bf16_round(v);
    ((uint16_t *)p)[idx] = h;
    return bf16_widen(h);
}

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as    */
/* easy as 1, 2, 3", SC'11).  Ten rounds; the key is bumped between rounds.   */
/* ------------------------------------------------------------------------- */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * The uniform of block `blk` (App. B.1: one eps ~ U[0,1) per block).  Four blocks share one
 * Philox call: counter = (blk/4 low, blk/4 high, stream, 0), key = seed, the block takes
 * output word blk%4 and its top 24 bits, so eps = u24 / 2^24 is exact in binary32.
 */
uint32_t oracle_block_u24(uint64_t seed, uint32_t stream_id, uint64_t blk)
{
    uint64_t c = blk >> 2;
    uint32_t ctr[4] = { (uint32_t)c, (uint32_t)(c >> 32), stream_id, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    return out[blk & 3u] >> 8;
}

static float u24_to_eps(uint32_t u24) { return (float)u24 * 0x1p-24f; }

/* ------------------------------------------------------------------------- */
/* MVUE 1:2 (Sec. 4.1, eq. (6)).                                              */
/*   keep a1 w.p. |a1|/(|a1|+|a2|) and emit sign(a1)(|a1|+|a2|); else a2.      */
/* Threshold form (App. B.1): keep a1 iff eps < p1, evaluated without the     */
/* division as  eps*(|a1|+|a2|) < |a1|.  A zero is never preferred to a        */
/* non-zero partner (p in {0,1}); an all-zero pair keeps position 0.           */
/* ------------------------------------------------------------------------- */
void oracle_select_1of2(const float x[2], float eps, int *kept, float *value)
{
    float m0 = fabsf(x[0]), m1 = fabsf(x[1]);
    float s = m0 + m1;
    float t = eps * s;
    int k = (m1 == 0.0f || t < m0) ? 0 : 1;
    *kept = k;
    *value = copysignf(s, x[k]);
}

/* ------------------------------------------------------------------------- */
/* optimal MVUE 2:4 (Sec. 4.2 + App. A.2).                                    */
/* Magnitudes are ranked a1<=a2<=a3<=a4 (the appendix assumes this order      */
/* w.l.o.g.); among equal magnitudes the element at the higher position ranks  */
/* lower.  One eps walks the cumulative pair probabilities in the order        */
/* p13,p14,p23,p24,p34 (p12 = 0 in every case):                                */
/*   case 1  a4 <= 2a1+a3 ........ denominators 2(a1+a2+a3+a4)                  */
/*   case 2  a4 <= a1+a2+a3 ...... same probabilities written over 2(a1+..+a4)  */
/*   case 3  otherwise ............ a4 kept w.p. 1, partner i w.p. a_i/(a1+a2+a3)*/
/* Kept magnitudes follow theta_i = a_i/p_i (eq. (8)): with p_i = 2a_i/sum     */
/* (eq. (12)) that is sum/2; in case 3 (eq. (14)) a4 is unchanged and the      */
/* partner becomes a1+a2+a3.  Signs are those of the inputs.                   */
/* ------------------------------------------------------------------------- */
void oracle_select_2of4(const float x[4], float eps, int pos[2], float value[2], int *which_case)
{
    /* rank: insertion sort on (magnitude asc, position desc) */
    int r[4] = { 3, 2, 1, 0 };           /* already "position descending" for all-equal */
    float m[4];
    for (int i = 0; i < 4; ++i) m[i] = fabsf(x[i]);
    for (int i = 1; i < 4; ++i) {
        int cur = r[i], j = i - 1;
        while (j >= 0 && m[r[j]] > m[cur]) { r[j + 1] = r[j]; --j; }
        r[j + 1] = cur;
    }
    const float a1 = m[r[0]], a2 = m[r[1]], a3 = m[r[2]], a4 = m[r[3]];
    const float s12 = a1 + a2;
    const float s123 = s12 + a3;
    const float s = s123 + a4;

    int ra, rb;            /* ranks (0-based) of the kept pair, ra < rb */
    float va, vb;          /* their output magnitudes */
    const float two_a1_a3 = 2.0f * a1 + a3;
    if (a4 <= two_a1_a3 || a4 <= s123) {
        const int c1case = (a4 <= two_a1_a3);
        const float t = eps * (2.0f * s);
        const float c13 = c1case ? (two_a1_a3 - a4) : 0.0f;              /* 2S*p13 */
        const float c14 = 4.0f * a1;                                     /* 2S*(p13+p14) */
        const float n23 = c1case ? ((2.0f * a2 + a3) - a4)               /* 2S*p23, case 1 */
                                 : (2.0f * (s123 - a4));                 /* 2S*p23, case 2 */
        const float c23 = c14 + n23;
        const float c24 = 4.0f * s12;                                    /* 2S*(1-p34) */
        if (t < c13)      { ra = 0; rb = 2; }
        else if (t < c14) { ra = 0; rb = 3; }
        else if (t < c23) { ra = 1; rb = 2; }
        else if (t < c24) { ra = 1; rb = 3; }
        else              { ra = 2; rb = 3; }
        va = vb = 0.5f * s;
        *which_case = c1case ? 1 : 2;
    } else {
        const float t = eps * s123;
        if (t < a1)       ra = 0;
        else if (t < s12) ra = 1;
        else              ra = 2;
        rb = 3;
        va = s123;
        vb = a4;
        *which_case = 3;
    }
    int pa = r[ra], pb = r[rb];
    float fa = copysignf(va, x[pa]), fb = copysignf(vb, x[pb]);
    if (pa < pb) { pos[0] = pa; pos[1] = pb; value[0] = fa; value[1] = fb; }
    else         { pos[0] = pb; pos[1] = pa; value[0] = fb; value[1] = fa; }
}

/*
 * The two uniforms of block `blk` for approx-MVUE 2:4 (Sec. 4.4 draws twice).  Two blocks share
 * one Philox call: counter = (blk/2 low, blk/2 high, stream, 1) -- the last word separates this
 * stream from the one-uniform-per-block stream above -- and the block takes output words
 * 2*(blk%2) and 2*(blk%2)+1, top 24 bits each.
 */
void oracle_block_u24_pair(uint64_t seed, uint32_t stream_id, uint64_t blk, uint32_t u[2])
{
    uint64_t c = blk >> 1;
    uint32_t ctr[4] = { (uint32_t)c, (uint32_t)(c >> 32), stream_id, 1u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    u[0] = out[2u * (blk & 1u)] >> 8;
    u[1] = out[2u * (blk & 1u) + 1u] >> 8;
}

/* ------------------------------------------------------------------------- */
/* approx-MVUE 2:4 (Sec. 4.4).                                                 */
/* One element is drawn with probability a_i / sum, a second one from the      */
/* remaining three with probability a_j / (sum - a_i); both are kept with the  */
/* value a_k / p_k, where p_k is the probability that k is one of the two      */
/* (the section's last equation):                                              */
/*     p_k = v_k (1 + sum_{l != k} v_l / (1 - v_l)),   v = a / sum             */
/* so  a_k / p_k = sum / (1 + sum_{l != k} a_l / (sum - a_l)).                 */
/* No ranking is needed: everything runs in position order.                    */
/*                                                                             */
/* Draw (threshold walk, no division): t = eps * total; the element is the     */
/* first position k whose running sum exceeds t.  If none does (possible only  */
/* through rounding, or when nothing non-zero is left) it is the last position */
/* with a non-zero magnitude, and if there is none, the lowest position not    */
/* taken yet -- so a zero is never drawn while a non-zero remains, and padding */
/* falls on the lowest-index zeros.  The second draw repeats the first on the  */
/* block with the drawn element's magnitude set to zero.                       */
/* "sum - a_l" is formed as the sum of the other three magnitudes (no          */
/* cancellation when one element dominates), and the sum over l != k likewise  */
/* (term k replaced by zero).  A zero magnitude contributes no term.           */
/* ------------------------------------------------------------------------- */
static int approx_draw(const float m[4], float eps, int taken)
{
    const float c0 = m[0], c1 = c0 + m[1], c2 = c1 + m[2], total = c2 + m[3];
    const float t = eps * total;
    if (t < c0) return 0;
    if (t < c1) return 1;
    if (t < c2) return 2;
    if (t < total) return 3;
    for (int k = 3; k >= 0; --k) if (m[k] > 0.0f) return k;
    for (int k = 0; k < 4; ++k) if (k != taken) return k;
    return 0;
}

void oracle_select_2of4_approx(const float x[4], float eps1, float eps2, int pos[2], float value[2])
{
    float m[4];
    for (int k = 0; k < 4; ++k) m[k] = fabsf(x[k]);
    const int i = approx_draw(m, eps1, -1);
    float r[4];
    for (int k = 0; k < 4; ++k) r[k] = (k == i) ? 0.0f : m[k];
    const int j = approx_draw(r, eps2, i);

    /* values */
    const float s01 = m[0] + m[1], s23 = m[2] + m[3];
    const float total = ((m[0] + m[1]) + m[2]) + m[3];
    const float others[4] = { m[1] + s23, m[0] + s23, s01 + m[3], s01 + m[2] };      /* sum - a_l, without cancellation */
    float vv[4];
    for (int l = 0; l < 4; ++l) vv[l] = (m[l] > 0.0f) ? m[l] / others[l] : 0.0f;     /* v_l / (1 - v_l) */
    float out[2];
    const int kept[2] = { i, j };
    for (int e = 0; e < 2; ++e) {
        const int k = kept[e];
        float z[4];
        for (int l = 0; l < 4; ++l) z[l] = (l == k) ? 0.0f : vv[l];
        const float denom = 1.0f + (((z[0] + z[1]) + z[2]) + z[3]);
        out[e] = copysignf(total / denom, x[k]);
    }
    if (i < j) { pos[0] = i; pos[1] = j; value[0] = out[0]; value[1] = out[1]; }
    else       { pos[0] = j; pos[1] = i; value[0] = out[1]; value[1] = out[0]; }
}

/* ------------------------------------------------------------------------- */
/* exhaustive enumeration over all 2^24 thresholds (test support)              */
/* ------------------------------------------------------------------------- */
/* counts[k]: how many u24 keep position k; mean[k]: average output at position k (binary64). */
void oracle_enumerate_1of2(const float x[2], uint64_t counts[2], double mean[2], double second[2])
{
    counts[0] = counts[1] = 0; mean[0] = mean[1] = 0; second[0] = second[1] = 0;
    for (uint32_t u = 0; u < (1u << 24); ++u) {
        int k; float v;
        oracle_select_1of2(x, u24_to_eps(u), &k, &v);
        counts[k] += 1; mean[k] += (double)v; second[k] += (double)v * (double)v;
    }
    for (int k = 0; k < 2; ++k) { mean[k] /= 16777216.0; second[k] /= 16777216.0; }
}

/* pair_counts[6] in the order (0,1),(0,2),(0,3),(1,2),(1,3),(2,3) of *positions*. */
void oracle_enumerate_2of4(const float x[4], uint64_t pair_counts[6], double mean[4], double second[4])
{
    static const int pair_id[4][4] = { {-1,0,1,2}, {0,-1,3,4}, {1,3,-1,5}, {2,4,5,-1} };
    for (int i = 0; i < 6; ++i) pair_counts[i] = 0;
    for (int i = 0; i < 4; ++i) { mean[i] = 0; second[i] = 0; }
    for (uint32_t u = 0; u < (1u << 24); ++u) {
        int pos[2], wc; float v[2];
        oracle_select_2of4(x, u24_to_eps(u), pos, v, &wc);
        pair_counts[pair_id[pos[0]][pos[1]]] += 1;
        for (int s = 0; s < 2; ++s) { mean[pos[s]] += (double)v[s]; second[pos[s]] += (double)v[s] * (double)v[s]; }
    }
    for (int i = 0; i < 4; ++i) { mean[i] /= 16777216.0; second[i] /= 16777216.0; }
}

/* ------------------------------------------------------------------------- */
/* tensor-level prune + compress.  g is [T x O], row stride ldg (elements);    */
/* blocks run along T.  Block index for the random source:                     */
/*     blk = (t / M) * O + o     (M = 2 or 4; O = logical columns)              */
/* Outputs in the group format; `dense` (nullable) receives theta(g), [T x O]  */
/* with row stride ldd, pruned positions +0.                                    */
/* Returns 0, or -1 for shapes the format cannot hold (T % 16 != 0).            */
/* ------------------------------------------------------------------------- */
int oracle_prune_1of2(const void *g, int64_t T, int64_t O, int64_t ldg, int dt,
                      uint64_t seed, uint32_t stream_id,
                      void *vals, uint16_t *meta, void *dense, int64_t ldd)
{
    if (T % 16 || T < 0 || O < 0) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t G = 0; G < T / 16; ++G) {
        for (int64_t o = 0; o < O; ++o) {
            uint16_t md = 0;
            for (int i = 0; i < 4; ++i) {          /* quad i = pairs 2i, 2i+1 */
                for (int s = 0; s < 2; ++s) {
                    int64_t pr = G * 8 + i * 2 + s;           /* pair row */
                    int64_t t0 = pr * 2;
                    float x[2] = { load_elem(g, dt, t0 * ldg + o), load_elem(g, dt, (t0 + 1) * ldg + o) };
                    uint32_t u = oracle_block_u24(seed, stream_id, (uint64_t)pr * (uint64_t)O + (uint64_t)o);
                    int k; float v;
                    oracle_select_1of2(x, u24_to_eps(u), &k, &v);
                    float stored = store_elem(vals, dt, (G * O + o) * 8 + 2 * i + s, v);
                    md |= (uint16_t)((2 * s + k) << (4 * i + 2 * s));
                    if (dense) {
                        store_elem(dense, dt, (t0 + k) * ldd + o, stored);
                        store_elem(dense, dt, (t0 + 1 - k) * ldd + o, 0.0f);
                    }
                }
            }
            meta[G * O + o] = md;
        }
    }
    return 0;
}

int oracle_prune_2of4(const void *g, int64_t T, int64_t O, int64_t ldg, int dt,
                      uint64_t seed, uint32_t stream_id,
                      void *vals, uint16_t *meta, void *dense, int64_t ldd)
{
    if (T % 16 || T < 0 || O < 0) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t G = 0; G < T / 16; ++G) {
        for (int64_t o = 0; o < O; ++o) {
            uint16_t md = 0;
            for (int i = 0; i < 4; ++i) {
                int64_t q = G * 4 + i, t0 = q * 4;
                float x[4];
                for (int k = 0; k < 4; ++k) x[k] = load_elem(g, dt, (t0 + k) * ldg + o);
                uint32_t u = oracle_block_u24(seed, stream_id, (uint64_t)q * (uint64_t)O + (uint64_t)o);
                int pos[2], wc; float v[2];
                oracle_select_2of4(x, u24_to_eps(u), pos, v, &wc);
                float st0 = store_elem(vals, dt, (G * O + o) * 8 + 2 * i + 0, v[0]);
                float st1 = store_elem(vals, dt, (G * O + o) * 8 + 2 * i + 1, v[1]);
                md |= (uint16_t)((pos[0] | (pos[1] << 2)) << (4 * i));
                if (dense) {
                    for (int k = 0; k < 4; ++k) store_elem(dense, dt, (t0 + k) * ldd + o, 0.0f);
                    store_elem(dense, dt, (t0 + pos[0]) * ldd + o, st0);
                    store_elem(dense, dt, (t0 + pos[1]) * ldd + o, st1);
                }
            }
            meta[G * O + o] = md;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* MVUE 1:4 (appendix, additional sparsity results: the 1:2 estimator on a    */
/* larger block).  The argument of Sec. 4.1 with one survivor out of four:     */
/* unbiasedness forces the kept value a_i/p_i, and sum_i a_i^2/p_i under       */
/* sum_i p_i = 1 is smallest at p_i = |a_i|/sum|a|, which makes every kept     */
/* value sign(a_i) * sum|a| (eq. (6) with four terms).                         */
/* Var = sum_i |a_i| (sum|a| - |a_i|).                                          */
/* Threshold walk in position order as for the draws above (a zero is never    */
/* kept while a non-zero exists; an all-zero quad keeps position 0).           */
/* Stored in the 2:4 group format: the second slot of the quad is a +0 at the  */
/* lowest other position -- the padding nm_compress would choose.              */
/* ------------------------------------------------------------------------- */
void oracle_select_1of4(const float x[4], float eps, int *kept, float *value)
{
    float m[4];
    for (int k = 0; k < 4; ++k) m[k] = fabsf(x[k]);
    int k = approx_draw(m, eps, -1);
    float total = ((m[0] + m[1]) + m[2]) + m[3];
    *kept = k;
    *value = copysignf(total, x[k]);
}

void oracle_enumerate_1of4(const float x[4], uint64_t counts[4], double mean[4], double second[4])
{
    for (int k = 0; k < 4; ++k) { counts[k] = 0; mean[k] = 0.0; second[k] = 0.0; }
    for (uint32_t u = 0; u < (1u << 24); ++u) {
        int k; float v;
        oracle_select_1of4(x, u24_to_eps(u), &k, &v);
        counts[k] += 1; mean[k] += (double)v; second[k] += (double)v * (double)v;
    }
    for (int k = 0; k < 4; ++k) { mean[k] /= 16777216.0; second[k] /= 16777216.0; }
}

int oracle_prune_1of4(const void *g, int64_t T, int64_t O, int64_t ldg, int dt,
                      uint64_t seed, uint32_t stream_id,
                      void *vals, uint16_t *meta, void *dense, int64_t ldd)
{
    if (T % 16 || T < 0 || O < 0) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t G = 0; G < T / 16; ++G) {
        for (int64_t o = 0; o < O; ++o) {
            uint16_t md = 0;
            for (int i = 0; i < 4; ++i) {
                int64_t q = G * 4 + i, t0 = q * 4;
                float x[4];
                for (int k = 0; k < 4; ++k) x[k] = load_elem(g, dt, (t0 + k) * ldg + o);
                uint32_t u = oracle_block_u24(seed, stream_id, (uint64_t)q * (uint64_t)O + (uint64_t)o);
                int k; float v;
                oracle_select_1of4(x, u24_to_eps(u), &k, &v);
                int pad = (k == 0) ? 1 : 0;
                int pos0 = k < pad ? k : pad, pos1 = k < pad ? pad : k;
                float st0 = store_elem(vals, dt, (G * O + o) * 8 + 2 * i + 0, pos0 == k ? v : 0.0f);
                float st1 = store_elem(vals, dt, (G * O + o) * 8 + 2 * i + 1, pos1 == k ? v : 0.0f);
                md |= (uint16_t)((pos0 | (pos1 << 2)) << (4 * i));
                if (dense) {
                    for (int kk = 0; kk < 4; ++kk) store_elem(dense, dt, (t0 + kk) * ldd + o, 0.0f);
                    store_elem(dense, dt, (t0 + pos0) * ldd + o, st0);
                    store_elem(dense, dt, (t0 + pos1) * ldd + o, st1);
                }
            }
            meta[G * O + o] = md;
        }
    }
    return 0;
}

/* approx-MVUE test support: how often each position is drawn over all 2^24 uniforms.          */
/* first < 0: the first draw on |x|; otherwise the second draw given that `first` was drawn.   */
void oracle_enumerate_approx_draw(const float x[4], int first, uint64_t counts[4])
{
    float m[4];
    for (int k = 0; k < 4; ++k) { m[k] = (k == first) ? 0.0f : fabsf(x[k]); counts[k] = 0; }
    for (uint32_t u = 0; u < (1u << 24); ++u) counts[approx_draw(m, u24_to_eps(u), first)] += 1;
}

int oracle_prune_2of4_approx(const void *g, int64_t T, int64_t O, int64_t ldg, int dt,
                             uint64_t seed, uint32_t stream_id,
                             void *vals, uint16_t *meta, void *dense, int64_t ldd)
{
    if (T % 16 || T < 0 || O < 0) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t G = 0; G < T / 16; ++G) {
        for (int64_t o = 0; o < O; ++o) {
            uint16_t md = 0;
            for (int i = 0; i < 4; ++i) {
                int64_t q = G * 4 + i, t0 = q * 4;
                float x[4];
                for (int k = 0; k < 4; ++k) x[k] = load_elem(g, dt, (t0 + k) * ldg + o);
                uint32_t u[2];
                oracle_block_u24_pair(seed, stream_id, (uint64_t)q * (uint64_t)O + (uint64_t)o, u);
                int pos[2]; float v[2];
                oracle_select_2of4_approx(x, u24_to_eps(u[0]), u24_to_eps(u[1]), pos, v);
                float st0 = store_elem(vals, dt, (G * O + o) * 8 + 2 * i + 0, v[0]);
                float st1 = store_elem(vals, dt, (G * O + o) * 8 + 2 * i + 1, v[1]);
                md |= (uint16_t)((pos[0] | (pos[1] << 2)) << (4 * i));
                if (dense) {
                    for (int k = 0; k < 4; ++k) store_elem(dense, dt, (t0 + k) * ldd + o, 0.0f);
                    store_elem(dense, dt, (t0 + pos[0]) * ldd + o, st0);
                    store_elem(dense, dt, (t0 + pos[1]) * ldd + o, st1);
                }
            }
            meta[G * O + o] = md;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* deterministic compression of a tensor that already is n:m sparse along T.   */
/* Kept positions = non-zero positions, padded with the lowest-index zero       */
/* positions of the block (pair for 1:2, quad for 2:4); values are copied       */
/* bit for bit.  Returns the number of blocks holding more than n non-zeros     */
/* (their output is unspecified), or -1 for a bad shape / (n,m).                */
/* ------------------------------------------------------------------------- */
int64_t oracle_nm_compress(const void *dense, int64_t T, int64_t O, int64_t ld, int dt, int n, int m,
                           void *vals, uint16_t *meta)
{
    if (T % 16 || !((n == 1 && m == 2) || (n == 2 && m == 4))) return -1;
    int64_t bad = 0;
    for (int64_t G = 0; G < T / 16; ++G) {
        for (int64_t o = 0; o < O; ++o) {
            uint16_t md = 0;
            for (int i = 0; i < 4; ++i) {
                int64_t t0 = (G * 4 + i) * 4;
                int keep[2], nk = 0;
                if (m == 4) {
                    int nzc = 0, taken[4] = {0, 0, 0, 0};
                    for (int k = 0; k < 4; ++k) if (load_elem(dense, dt, (t0 + k) * ld + o) != 0.0f) { taken[k] = 1; ++nzc; }
                    if (nzc > 2) ++bad;
                    for (int k = 0; k < 4 && nzc < 2; ++k) if (!taken[k]) { taken[k] = 1; ++nzc; }
                    for (int k = 0; k < 4 && nk < 2; ++k) if (taken[k]) keep[nk++] = k;
                } else {
                    for (int s = 0; s < 2; ++s) {
                        int z0 = load_elem(dense, dt, (t0 + 2 * s) * ld + o) != 0.0f;
                        int z1 = load_elem(dense, dt, (t0 + 2 * s + 1) * ld + o) != 0.0f;
                        if (z0 && z1) ++bad;
                        keep[nk++] = 2 * s + ((z1 && !z0) ? 1 : 0);
                    }
                }
                for (int s = 0; s < 2; ++s) {
                    int64_t src = (t0 + keep[s]) * ld + o, dst = (G * O + o) * 8 + 2 * i + s;
                    if (dt == DT_F32) ((float *)vals)[dst] = ((const float *)dense)[src];
                    else ((uint16_t *)vals)[dst] = ((const uint16_t *)dense)[src];
                }
                md |= (uint16_t)((keep[0] | (keep[1] << 2)) << (4 * i));
            }
            meta[G * O + o] = md;
        }
    }
    return bad;
}

/* expand the group format back to a dense [T x O] tensor (row stride ldd), pruned positions +0 */
void oracle_nm_decompress(const void *vals, const uint16_t *meta, int64_t T, int64_t O, int dt,
                          void *dense, int64_t ldd)
{
    for (int64_t G = 0; G < T / 16; ++G)
        for (int64_t o = 0; o < O; ++o) {
            uint16_t md = meta[G * O + o];
            for (int i = 0; i < 4; ++i) {
                int64_t t0 = (G * 4 + i) * 4;
                for (int k = 0; k < 4; ++k) {
                    int64_t dst = (t0 + k) * ldd + o;
                    if (dt == DT_F32) ((float *)dense)[dst] = 0.0f; else ((uint16_t *)dense)[dst] = 0;
                }
                for (int s = 0; s < 2; ++s) {
                    int k = (md >> (4 * i + 2 * s)) & 3;
                    int64_t src = (G * O + o) * 8 + 2 * i + s, dst = (t0 + k) * ldd + o;
                    if (dt == DT_F32) ((float *)dense)[dst] = ((const float *)vals)[src];
                    else ((uint16_t *)dense)[dst] = ((const uint16_t *)vals)[src];
                }
            }
        }
}

/* ------------------------------------------------------------------------- */
/* update GEMM, eq. (3), oriented [O x I]:                                      */
/*     dW[o][i] = beta*dW_in[o][i] + sum_t gt[t][o] * h[t][i]                    */
/* with gt the decompressed operand, every product and sum in binary64, t       */
/* ascending.  absdW[o][i] = sum_t |gt[t][o]| |h[t][i]| (the scale a rounding     */
/* error bound is stated against); nullable.                                     */
/* ------------------------------------------------------------------------- */
void oracle_update_gemm(const void *vals, const uint16_t *meta, const void *h, int64_t ldh,
                        int64_t T, int64_t O, int64_t I, int dt, double beta, const float *dW_in,
                        double *dW, double *absdW)
{
    #pragma omp parallel for schedule(dynamic, 4)
    for (int64_t o = 0; o < O; ++o) {
        double *row = dW + o * I, *arow = absdW ? absdW + o * I : NULL;
        for (int64_t i = 0; i < I; ++i) {
            row[i] = (beta != 0.0 && dW_in) ? beta * (double)dW_in[o * I + i] : 0.0;
            if (arow) arow[i] = 0.0;
        }
        for (int64_t t = 0; t < T; ++t) {
            /* element (t, o) of the decompressed operand */
            int64_t G = t / 16; int qi = (int)((t % 16) / 4), k = (int)(t % 4);
            uint16_t md = meta[G * O + o];
            double gv = 0.0;
            for (int s = 0; s < 2; ++s)
                if (((md >> (4 * qi + 2 * s)) & 3) == k)
                    gv = (double)load_elem(vals, dt, (G * O + o) * 8 + 2 * qi + s);
            for (int64_t i = 0; i < I; ++i) {
                double hv = (double)load_elem(h, dt, t * ldh + i);
                row[i] += gv * hv;
                if (arow) arow[i] += fabs(gv) * fabs(hv);
            }
        }
    }
}

/* the same sum for a list of n (o,i) entries: oi = {o0,i0,o1,i1,...} */
void oracle_update_gemm_entries(const void *vals, const uint16_t *meta, const void *h, int64_t ldh,
                                int64_t T, int64_t O, int64_t I, int dt,
                                const int64_t *oi, int64_t n, double *out, double *out_abs)
{
    (void)I;
    #pragma omp parallel for schedule(dynamic, 16)
    for (int64_t e = 0; e < n; ++e) {
        int64_t o = oi[2 * e], i = oi[2 * e + 1];
        double acc = 0.0, aacc = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            int64_t G = t / 16; int qi = (int)((t % 16) / 4), k = (int)(t % 4);
            uint16_t md = meta[G * O + o];
            double gv = 0.0;
            for (int s = 0; s < 2; ++s)
                if (((md >> (4 * qi + 2 * s)) & 3) == k)
                    gv = (double)load_elem(vals, dt, (G * O + o) * 8 + 2 * qi + s);
            double hv = (double)load_elem(h, dt, t * ldh + i);
            acc += gv * hv; aacc += fabs(gv) * fabs(hv);
        }
        out[e] = acc;
        if (out_abs) out_abs[e] = aacc;
    }
}

/* ------------------------------------------------------------------------- */
/* 8-bit neural gradients on top of 2:4 sparsity (Sec. 5, the "8-bit" rows of    */
/* the table that combines sparsity in all training phases with quantisation:    */
/* FP8 neural gradients).  Sec. 3 recalls why the quantiser of a neural gradient */
/* has to be unbiased: stochastic rounding.  The paper fixes neither the bit     */
/* layout nor the scale; this build takes                                         */
/*   gradients   e5m2 (1 sign, 5 exponent, 2 mantissa bits, bias 15, IEEE-like    */
/*               subnormals; the finite codes are the upper byte of a binary16)   */
/*   activations e4m3 (1-4-3, bias 7, no infinities, 0x7F/0xFF = NaN, max 448)    */
/*               -- the 8-bit format the matrix unit multiplies e5m2 with; it     */
/*               stands in for the paper's INT8 activations                       */
/* both as defined by the OCP 8-bit floating point specification (OFP8).          */
/* ------------------------------------------------------------------------- */
double oracle_e5m2_value(uint8_t c)
{
    int sign = c >> 7, e = (c >> 2) & 31, m = c & 3;
    double v;
    if (e == 31) v = m ? NAN : INFINITY;
    else if (e == 0) v = ldexp((double)m, -16);                 /* subnormal: m/4 * 2^-14 */
    else v = ldexp(1.0 + (double)m / 4.0, e - 15);
    return sign ? -v : v;
}

double oracle_e4m3_value(uint8_t c)
{
    int sign = c >> 7, e = (c >> 3) & 15, m = c & 7;
    double v;
    if (e == 15 && m == 7) v = NAN;
    else if (e == 0) v = ldexp((double)m, -9);                  /* subnormal: m/8 * 2^-6 */
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

/*
 * Stochastic rounding of a binary32 value to e5m2 with 16 random bits r16 in [0, 2^16).
 * lo <= |x| < hi are neighbouring magnitudes of the e5m2 grid and f = (|x| - lo)/(hi - lo):
 * the result is hi when  r16 + floor(f * 2^16) >= 2^16,  else lo; the sign is kept.  Over a
 * uniform r16 the mean is lo + (hi - lo) * floor(f 2^16) / 2^16: unbiased up to 2^-16 of a grid
 * step.  Magnitudes at or above the largest finite value (57344) saturate to it; NaN gives NaN.
 */
uint8_t oracle_sr_e5m2(float x, uint32_t r16)
{
    uint8_t sign = (uint8_t)(float_to_bits(x) >> 31 << 7);
    double m = fabs((double)x);
    if (isnan(x)) return (uint8_t)(sign | 0x7F);
    if (m >= oracle_e5m2_value(0x7B)) return (uint8_t)(sign | 0x7B);
    int c = 0;
    while (oracle_e5m2_value((uint8_t)(c + 1)) <= m) ++c;       /* codes 0..0x7B ascend with magnitude */
    double lo = oracle_e5m2_value((uint8_t)c), hi = oracle_e5m2_value((uint8_t)(c + 1));
    double f = (m - lo) / (hi - lo);
    uint32_t thr = (uint32_t)floor(f * 65536.0);
    return (uint8_t)(sign | (uint8_t)(c + ((r16 & 0xFFFFu) + thr >= 65536u ? 1 : 0)));
}

/*
 * The rounding bits of block `blk`: one Philox call per four blocks, counter = (blk/4 low, blk/4 high,
 * stream, 2) -- the last word separates this stream from the selection streams above --, the block
 * takes output word blk%4; its low half rounds the first kept value, its high half the second.
 */
void oracle_block_r16_pair(uint64_t seed, uint32_t stream_id, uint64_t blk, uint32_t r[2])
{
    uint64_t call = blk >> 2;
    uint32_t ctr[4] = { (uint32_t)call, (uint32_t)(call >> 32), stream_id, 2u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    r[0] = out[blk & 3] & 0xFFFFu;
    r[1] = out[blk & 3] >> 16;
}

/*
 * 2:4 prune (mode 0: optimal MVUE, Sec. 4.2; mode 1: approx-MVUE, Sec. 4.4) with 8-bit output.
 * Selection and kept values are exactly those of oracle_prune_2of4 / oracle_prune_2of4_approx
 * (same random stream, same block index), taken in binary32 before any storage rounding; each
 * kept value is multiplied by `scale` (one binary32 product) and rounded stochastically to e5m2.
 * E[q / scale] = theta(g) up to the 2^-16 granularity above, so the estimate stays unbiased (Sec. 3).
 *
 * 8-bit group format: groups of 32 tokens = 8 quads.  For group G and column o
 *     vals8[(G*O + o)*16 + 2*i + s]   s-th kept value (ascending position) of quad i, i = 0..7
 *     meta32[G*O + o]  (uint32)       bits [4i+1:4i] = position of kept 0, [4i+3:4i+2] = kept 1
 * Returns 0, or -1 for shapes the format cannot hold (T % 32 != 0) or an unknown mode.
 */
int oracle_prune_2of4_q8(const void *g, int64_t T, int64_t O, int64_t ldg, int dt,
                         uint64_t seed, uint32_t stream_id, int mode, float scale,
                         uint8_t *vals8, uint32_t *meta32)
{
    if (T % 32 || T < 0 || O < 0 || (mode != 0 && mode != 1)) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t G = 0; G < T / 32; ++G) {
        for (int64_t o = 0; o < O; ++o) {
            uint32_t md = 0;
            for (int i = 0; i < 8; ++i) {
                int64_t q = G * 8 + i, t0 = q * 4;
                uint64_t blk = (uint64_t)q * (uint64_t)O + (uint64_t)o;
                float x[4];
                for (int k = 0; k < 4; ++k) x[k] = load_elem(g, dt, (t0 + k) * ldg + o);
                int pos[2]; float v[2];
                if (mode == 0) {
                    int wc;
                    oracle_select_2of4(x, u24_to_eps(oracle_block_u24(seed, stream_id, blk)), pos, v, &wc);
                } else {
                    uint32_t u[2];
                    oracle_block_u24_pair(seed, stream_id, blk, u);
                    oracle_select_2of4_approx(x, u24_to_eps(u[0]), u24_to_eps(u[1]), pos, v);
                }
                uint32_t r[2];
                oracle_block_r16_pair(seed, stream_id, blk, r);
                for (int s = 0; s < 2; ++s) {
                    float scaled = v[s] * scale;
                    vals8[(G * O + o) * 16 + 2 * i + s] = oracle_sr_e5m2(scaled, r[s]);
                }
                md |= (uint32_t)(pos[0] | (pos[1] << 2)) << (4 * i);
            }
            meta32[G * O + o] = md;
        }
    }
    return 0;
}

/*
 * MVUE 1:2 prune (Sec. 4.1, eq. (6)) with 8-bit output, in the same 8-bit group format: quad i of a group holds
 * the pairs 2i and 2i+1; the kept value of the first pair (position 0 or 1) is slot 2i, that of the second
 * (position 2 or 3) slot 2i+1.  Selection and value are those of oracle_prune_1of2 (same random stream, block
 * index = pair row * O + column), taken in binary32 before any storage rounding; the value is multiplied by
 * `scale` and rounded stochastically to e5m2 with the LOW half of the pair block's rounding word
 * (oracle_block_r16_pair with the pair's block index).
 */
int oracle_prune_1of2_q8(const void *g, int64_t T, int64_t O, int64_t ldg, int dt,
                         uint64_t seed, uint32_t stream_id, float scale, uint8_t *vals8, uint32_t *meta32)
{
    if (T % 32 || T < 0 || O < 0) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t G = 0; G < T / 32; ++G) {
        for (int64_t o = 0; o < O; ++o) {
            uint32_t md = 0;
            for (int p = 0; p < 16; ++p) {                 /* pair p of the group: tokens 32G + 2p, 32G + 2p + 1 */
                int64_t pr = G * 16 + p, t0 = pr * 2;
                uint64_t blk = (uint64_t)pr * (uint64_t)O + (uint64_t)o;
                float x[2] = { load_elem(g, dt, t0 * ldg + o), load_elem(g, dt, (t0 + 1) * ldg + o) };
                int k; float v;
                oracle_select_1of2(x, u24_to_eps(oracle_block_u24(seed, stream_id, blk)), &k, &v);
                uint32_t r[2];
                oracle_block_r16_pair(seed, stream_id, blk, r);
                vals8[(G * O + o) * 16 + p] = oracle_sr_e5m2(v * scale, r[0]);
                md |= (uint32_t)(((p & 1) << 1) | k) << (2 * p);
            }
            meta32[G * O + o] = md;
        }
    }
    return 0;
}

/* expand the 8-bit group format to a dense binary64 [T x O] tensor (decoded e5m2 values, pruned positions 0) */
void oracle_nm_decompress_q8(const uint8_t *vals8, const uint32_t *meta32, int64_t T, int64_t O, double *dense)
{
    for (int64_t t = 0; t < T; ++t)
        for (int64_t o = 0; o < O; ++o) dense[t * O + o] = 0.0;
    for (int64_t G = 0; G < T / 32; ++G)
        for (int64_t o = 0; o < O; ++o)
            for (int i = 0; i < 8; ++i)
                for (int s = 0; s < 2; ++s) {
                    int k = (int)((meta32[G * O + o] >> (4 * i + 2 * s)) & 3u);
                    dense[(G * 32 + 4 * i + k) * O + o] = oracle_e5m2_value(vals8[(G * O + o) * 16 + 2 * i + s]);
                }
}

/*
 * Update GEMM (eq. (3)) on the 8-bit operands, for n entries oi = {o0,i0,o1,i1,...} (n = O*I with
 * oi == NULL means every entry, row-major):
 *     out = alpha * sum_t e5m2(gt[t][o]) * e4m3(h8[t][i])        (binary64, t ascending)
 * alpha undoes the two scales (1 / (scale_g * scale_h)).  out_abs: the same sum over magnitudes.
 */
void oracle_update_gemm_q8(const uint8_t *vals8, const uint32_t *meta32, const uint8_t *h8, int64_t ldh,
                           int64_t T, int64_t O, int64_t I, double alpha,
                           const int64_t *oi, int64_t n, double *out, double *out_abs)
{
    #pragma omp parallel for schedule(dynamic, 16)
    for (int64_t e = 0; e < n; ++e) {
        int64_t o = oi ? oi[2 * e] : e / I, i = oi ? oi[2 * e + 1] : e % I;
        double acc = 0.0, aacc = 0.0;
        (void)O;
        for (int64_t t = 0; t < T; ++t) {
            int64_t G = t / 32; int qi = (int)((t % 32) / 4), k = (int)(t % 4);
            uint32_t md = meta32[G * O + o];
            double gv = 0.0;
            for (int s = 0; s < 2; ++s)
                if ((int)((md >> (4 * qi + 2 * s)) & 3u) == k)
                    gv = oracle_e5m2_value(vals8[(G * O + o) * 16 + 2 * qi + s]);
            double hv = oracle_e4m3_value(h8[t * ldh + i]);
            acc += gv * hv; aacc += fabs(gv) * fabs(hv);
        }
        out[e] = alpha * acc;
        if (out_abs) out_abs[e] = fabs(alpha) * aacc;
    }
}

/* ------------------------------------------------------------------------- */
/* Update GEMM of a convolution without the im2col matrix (App. B.1, part 1:   */
/* activation A [B x C_I x H x W], gradients G [B x C_O x H x W], update Delta  */
/* [C_I x C_O x k x k]).  Stated on rows: x is a [rows x C] matrix (the zero-   */
/* padded channels-last activation grid, flattened), gt the decompressed       */
/* gradient on the same grid, and kernel tap j pairs output row t with input    */
/* row t + shift[j]:                                                            */
/*     dW[o][j*C + c] = sum_t gt[t][o] * x[(t + shift[j])*ldx + c]   (binary64)  */
/* x points at row 0; rows -margin .. T+margin-1 must exist, margin >= |shift|. */
/* ------------------------------------------------------------------------- */
void oracle_update_gemm_shifted(const void *vals, const uint16_t *meta, const void *x, int64_t ldx, int64_t C,
                                const int64_t *shift, int n_shift, int64_t T, int64_t O, int dt,
                                double *dW, double *absdW)
{
    const int64_t I = (int64_t)n_shift * C;
    #pragma omp parallel for schedule(dynamic, 4)
    for (int64_t o = 0; o < O; ++o) {
        double *row = dW + o * I, *arow = absdW ? absdW + o * I : NULL;
        for (int64_t i = 0; i < I; ++i) { row[i] = 0.0; if (arow) arow[i] = 0.0; }
        for (int64_t t = 0; t < T; ++t) {
            int64_t G = t / 16; int qi = (int)((t % 16) / 4), k = (int)(t % 4);
            uint16_t md = meta[G * O + o];
            double gv = 0.0;
            for (int s = 0; s < 2; ++s)
                if (((md >> (4 * qi + 2 * s)) & 3) == k)
                    gv = (double)load_elem(vals, dt, (G * O + o) * 8 + 2 * qi + s);
            if (gv == 0.0) continue;
            for (int j = 0; j < n_shift; ++j)
                for (int64_t c = 0; c < C; ++c) {
                    double hv = (double)load_elem(x, dt, (t + shift[j]) * ldx + c);
                    row[j * C + c] += gv * hv;
                    if (arow) arow[j * C + c] += fabs(gv) * fabs(hv);
                }
        }
    }
}

/* the 8-bit form of the same product: dW[o][j*C + c] = alpha * sum_t e5m2(gt[t][o]) * e4m3(x8[(t + shift[j])*ldx + c]) */
void oracle_update_gemm_q8_shifted(const uint8_t *vals8, const uint32_t *meta32, const uint8_t *x8, int64_t ldx, int64_t C,
                                   const int64_t *shift, int n_shift, int64_t T, int64_t O, double alpha,
                                   double *dW, double *absdW)
{
    const int64_t I = (int64_t)n_shift * C;
    #pragma omp parallel for schedule(dynamic, 4)
    for (int64_t o = 0; o < O; ++o) {
        double *row = dW + o * I, *arow = absdW ? absdW + o * I : NULL;
        for (int64_t i = 0; i < I; ++i) { row[i] = 0.0; if (arow) arow[i] = 0.0; }
        for (int64_t t = 0; t < T; ++t) {
            int64_t G = t / 32; int qi = (int)((t % 32) / 4), k = (int)(t % 4);
            uint32_t md = meta32[G * O + o];
            double gv = 0.0;
            for (int s = 0; s < 2; ++s)
                if ((int)((md >> (4 * qi + 2 * s)) & 3u) == k)
                    gv = oracle_e5m2_value(vals8[(G * O + o) * 16 + 2 * qi + s]);
            if (gv == 0.0) continue;
            for (int j = 0; j < n_shift; ++j)
                for (int64_t c = 0; c < C; ++c) {
                    double hv = oracle_e4m3_value(x8[(t + shift[j]) * ldx + c]);
                    row[j * C + c] += gv * hv;
                    if (arow) arow[j * C + c] += fabs(gv) * fabs(hv);
                }
        }
        for (int64_t i = 0; i < I; ++i) { row[i] *= alpha; if (arow) arow[i] *= fabs(alpha); }
    }
}

/* ------------------------------------------------------------------------- */
/* Per-tensor scale and the activations' 8-bit cast for the 8-bit path (Sec. 5,  */
/* 8-bit rows; the paper gives no scale rule).  Reading: one power-of-two scale  */
/* per tensor from its current maximum magnitude, the largest s = 2^e with       */
/* s * max|t| <= top (a power of two multiplies without rounding, so the scale   */
/* itself adds no error); e is kept in [-126, 126] so that s and 1/s are normal  */
/* binary32 numbers; an all-zero tensor, or one whose maximum is not finite,     */
/* gets s = 1.  `top` is the largest magnitude the 8-bit format may be asked to  */
/* hold: 448 for e4m3 activations, 57344 / 4 (2:4) or 57344 / 2 (1:2) for e5m2   */
/* gradients, whose kept values are at most the sum of their block's magnitudes. */
/* ------------------------------------------------------------------------- */
float oracle_pow2_scale(const void *t, int64_t R, int64_t C, int64_t ld, int dt, float top)
{
    /* the maximum over the bit patterns of |t|: they order like the magnitudes, with infinity and every NaN on top */
    uint32_t mb = 0;
    for (int64_t r = 0; r < R; ++r)
        for (int64_t c = 0; c < C; ++c) {
            uint32_t b = float_to_bits(load_elem(t, dt, r * ld + c)) & 0x7FFFFFFFu;
            if (b > mb) mb = b;
        }
    const float m = bits_to_float(mb);
    if (mb == 0 || mb >= 0x7F800000u || !(top > 0.0f) || !isfinite(top)) return 1.0f;
    int em, et;
    double fm = frexp((double)m, &em), ft = frexp((double)top, &et);      /* x = f * 2^e, f in [0.5, 1) */
    int e = et - em - (ft >= fm ? 0 : 1);                                  /* largest e with 2^e * m <= top */
    if (e > 126) e = 126;
    if (e < -126) e = -126;
    return (float)ldexp(1.0, e);
}

/* binary32 -> e4m3 (OCP), round to nearest, ties to even; magnitudes above 448 saturate to 448; NaN -> 0x7F */
uint8_t oracle_e4m3_rne(float x)
{
    uint8_t sign = (uint8_t)(float_to_bits(x) >> 31 << 7);
    if (isnan(x)) return (uint8_t)(sign | 0x7F);
    double m = fabs((double)x);
    if (m >= 448.0) return (uint8_t)(sign | 0x7E);
    int c = 0;
    while (c < 0x7E && oracle_e4m3_value((uint8_t)(c + 1)) <= m) ++c;       /* codes 0..0x7E ascend with magnitude */
    double lo = oracle_e4m3_value((uint8_t)c), hi = oracle_e4m3_value((uint8_t)(c + 1));
    double dl = m - lo, dh = hi - m;
    if (dh < dl || (dh == dl && (c & 1))) ++c;                               /* nearest; a tie goes to the even code */
    return (uint8_t)(sign | (uint8_t)c);
}

/* h8[r][c] = e4m3(fl(h[r][c] * scale)): one binary32 product, then the rounding above */
void oracle_cast_e4m3(const void *h, int64_t R, int64_t C, int64_t ld, int dt, float scale, uint8_t *h8, int64_t ld8)
{
    #pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r)
        for (int64_t c = 0; c < C; ++c) h8[r * ld8 + c] = oracle_e4m3_rne(load_elem(h, dt, r * ld + c) * scale);
}

/* ------------------------------------------------------------------------- */
/* The producer of the neural gradient (eq. (2)): g_l = Diag(f'(z_l)) W^T g_{l+1}. */
/* The matrix product u = W^T g_{l+1} is a dense GEMM the method leaves alone;     */
/* the last step that makes g_l is the elementwise product with the activation's  */
/* derivative d = f'(z_l).  Plain definition: one binary32 product per element,   */
/* rounded to the storage type -- that rounded tensor is the neural gradient the  */
/* next layer's backward GEMM reads and the prune of this layer's update phase    */
/* applies to.                                                                    */
/* ------------------------------------------------------------------------- */
void oracle_act_backward(const void *u, int64_t ldu, const void *d, int64_t ldd, int64_t T, int64_t O, int dt,
                         void *g, int64_t ldg)
{
    #pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int64_t o = 0; o < O; ++o)
            store_elem(g, dt, t * ldg + o, load_elem(u, dt, t * ldu + o) * load_elem(d, dt, t * ldd + o));
}

/* ------------------------------------------------------------------------- */
/* Greedy N:M (the "Greedy" rows of the 1:2 ablation table in Sec. 4.1 and of   */
/* the result tables in Sec. 5): keep the n largest magnitudes of the block,    */
/* values unchanged.  Deterministic and biased -- the comparison method, not    */
/* an estimator of this paper.  Among equal magnitudes the lower position is    */
/* kept (the ranking of the optimal 2:4 estimator above: of equal magnitudes    */
/* the element at the higher position ranks lower).                             */
/* pos[] comes back in ascending order.                                         */
/* ------------------------------------------------------------------------- */
void oracle_select_greedy(const float *x, int m, int n, int *pos)
{
    int taken[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int s = 0; s < n; ++s) {
        int best = -1;
        for (int k = 0; k < m; ++k)
            if (!taken[k] && (best < 0 || fabsf(x[k]) > fabsf(x[best]))) best = k;     /* strict: the first (lowest) wins a tie */
        taken[best] = 1;
    }
    int c = 0;
    for (int k = 0; k < m; ++k) if (taken[k]) pos[c++] = k;
}

/* tensor level, group format; (n, m) = (1, 2) or (2, 4).  Values are copied bit for bit. */
int oracle_prune_greedy(const void *g, int64_t T, int64_t O, int64_t ldg, int dt, int n, int m,
                        void *vals, uint16_t *meta, void *dense, int64_t ldd)
{
    if (T % 16 || T < 0 || O < 0 || !((n == 1 && m == 2) || (n == 2 && m == 4))) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t G = 0; G < T / 16; ++G) {
        for (int64_t o = 0; o < O; ++o) {
            uint16_t md = 0;
            for (int i = 0; i < 4; ++i) {
                int64_t t0 = (G * 4 + i) * 4;
                float x[4];
                for (int k = 0; k < 4; ++k) x[k] = load_elem(g, dt, (t0 + k) * ldg + o);
                int pos[2];
                if (m == 4) oracle_select_greedy(x, 4, 2, pos);
                else {                                   /* the quad holds two pairs */
                    oracle_select_greedy(x, 2, 1, &pos[0]);
                    oracle_select_greedy(x + 2, 2, 1, &pos[1]);
                    pos[1] += 2;
                }
                float st0 = store_elem(vals, dt, (G * O + o) * 8 + 2 * i + 0, x[pos[0]]);
                float st1 = store_elem(vals, dt, (G * O + o) * 8 + 2 * i + 1, x[pos[1]]);
                md |= (uint16_t)((pos[0] | (pos[1] << 2)) << (4 * i));
                if (dense) {
                    for (int k = 0; k < 4; ++k) store_elem(dense, dt, (t0 + k) * ldd + o, 0.0f);
                    store_elem(dense, dt, (t0 + pos[0]) * ldd + o, st0);
                    store_elem(dense, dt, (t0 + pos[1]) * ldd + o, st1);
                }
            }
            meta[G * O + o] = md;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* approx-MVUE 4:8 (appendix, "Additional sparsity results": the approximate    */
/* 2:4 method of Sec. 4.4 carried over to more elements).  Four elements of a   */
/* block of eight are drawn one after the other without replacement, each with  */
/* probability a_j / (sum of the magnitudes not yet drawn); every drawn element */
/* is kept with the value a_k / p_k, p_k = the probability that k is among the  */
/* four (the unbiasedness argument of Sec. 4.2, eq. (8)).                        */
/*                                                                             */
/* p_k has no short closed form for four draws.  It is computed from the        */
/* definition, organised by the SET of elements drawn so far (the next draw     */
/* depends on that set only): with f(U) the probability that the first |U|      */
/* draws are exactly the set U,                                                 */
/*     f({}) = 1,   f(U) = sum_{k in U} f(U \ k) * a_k / rest(U \ k),            */
/*     rest(V) = sum of the magnitudes outside V,   p_k = sum_{|U|=4, k in U} f(U). */
/* Pinned arithmetic (binary32, one rounding per operation):                    */
/*     rest(V) = lo(V) + hi(V), lo / hi = the sums of the magnitudes outside V   */
/*               among positions 0-3 / 4-7, each added in ascending position     */
/*               (never by subtraction: no cancellation when one element carries */
/*               the sum);                                                       */
/*     g(V) = f(V) / rest(V)   (IEEE division);                                  */
/*     f(U) = sum over k in U, ascending position, of g(U \ k) * a_k;            */
/*     p_k  = sum over the 4-sets U containing k in ascending order of their     */
/*            bit mask (bit j = position j).                                     */
/* A block with at most four non-zero magnitudes keeps all of them unchanged    */
/* (p = 1) and pads with its lowest-index zeros.  Otherwise every draw finds a  */
/* non-zero element, rest() is positive wherever it is used, and the value is   */
/* min(a_k / p_k, sum): in exact arithmetic a_k / p_k <= sum (the first draw     */
/* alone gives p_k >= a_k / sum), so the bound only acts on rounding.            */
/*                                                                             */
/* Draw: the threshold walk of the 2:4 method over eight positions (t = eps *   */
/* remaining total; first position whose running sum exceeds t; else the last   */
/* position with a non-zero magnitude left; else the lowest position not taken).*/
/* Four uniforms per block: one Philox call, counter = (blk low, blk high,      */
/* stream, 3), blk = (t / 8) * O + o, draw d takes the top 24 bits of word d.   */
/*                                                                             */
/* Compressed form (gfx950's sparse matrix instructions are 4:2 only, so this   */
/* is a storage format, not a GEMM operand): per 16-token group and column,     */
/*     vals[(G*O + o)*8 + 4*b + s]   s-th kept value (ascending position) of     */
/*                                   octet b = 0, 1 of the group                 */
/*     meta32[G*O + o]  (uint32)     bits [16b + 3s + 2 : 16b + 3s] = position    */
/*                                   (0..7) of kept value s of octet b            */
/* ------------------------------------------------------------------------- */
void oracle_block_u24_quad(uint64_t seed, uint32_t stream_id, uint64_t blk, uint32_t u[4])
{
    uint32_t ctr[4] = { (uint32_t)blk, (uint32_t)(blk >> 32), stream_id, 3u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    for (int d = 0; d < 4; ++d) u[d] = out[d] >> 8;
}

/* one draw among eight positions; m[] holds 0 at the positions already drawn, `taken` is their bit mask */
int oracle_draw8(const float m[8], float eps, unsigned taken)
{
    float run[8];
    run[0] = m[0];
    for (int k = 1; k < 8; ++k) run[k] = run[k - 1] + m[k];
    const float t = eps * run[7];
    for (int k = 0; k < 8; ++k) if (t < run[k]) return k;
    for (int k = 7; k >= 0; --k) if (m[k] > 0.0f) return k;
    for (int k = 0; k < 8; ++k) if (!((taken >> k) & 1u)) return k;
    return 0;
}

static int popcount8(unsigned v) { int c = 0; for (int k = 0; k < 8; ++k) c += (int)((v >> k) & 1u); return c; }

/* inclusion probabilities of four successive magnitude-proportional draws out of eight (needs >= 5 non-zeros) */
void oracle_inclusion_4of8(const float m[8], float p[8])
{
    static float f[256], g[256];
    #pragma omp threadprivate(f, g)
    for (int size = 0; size <= 4; ++size) {
        for (unsigned U = 0; U < 256; ++U) {
            if (popcount8(U) != size) continue;
            if (size == 0) f[U] = 1.0f;
            else {
                float acc = 0.0f;
                int first = 1;
                for (int k = 0; k < 8; ++k) {
                    if (!((U >> k) & 1u)) continue;
                    const float term = g[U & ~(1u << k)] * m[k];
                    acc = first ? term : acc + term;
                    first = 0;
                }
                f[U] = acc;
            }
            if (size < 4) {
                float lo = 0.0f, hi = 0.0f;
                int flo = 1, fhi = 1;
                for (int k = 0; k < 4; ++k) if (!((U >> k) & 1u)) { lo = flo ? m[k] : lo + m[k]; flo = 0; }
                for (int k = 4; k < 8; ++k) if (!((U >> k) & 1u)) { hi = fhi ? m[k] : hi + m[k]; fhi = 0; }
                g[U] = f[U] / (lo + hi);
            }
        }
    }
    for (int k = 0; k < 8; ++k) {
        float acc = 0.0f;
        int first = 1;
        for (unsigned U = 0; U < 256; ++U) {
            if (popcount8(U) != 4 || !((U >> k) & 1u)) continue;
            acc = first ? f[U] : acc + f[U];
            first = 0;
        }
        p[k] = acc;
    }
}

/* pos[] ascending, value[] in the same order */
void oracle_select_4of8_approx(const float x[8], const float eps[4], int pos[4], float value[4])
{
    float m[8], r[8];
    int nz = 0;
    for (int k = 0; k < 8; ++k) { m[k] = fabsf(x[k]); r[k] = m[k]; nz += m[k] > 0.0f; }
    unsigned taken = 0;
    for (int d = 0; d < 4; ++d) {
        const int k = oracle_draw8(r, eps[d], taken);
        taken |= 1u << k;
        r[k] = 0.0f;
    }
    float p[8];
    float total = 0.0f;
    if (nz > 4) {
        oracle_inclusion_4of8(m, p);
        const float lo = ((m[0] + m[1]) + m[2]) + m[3], hi = ((m[4] + m[5]) + m[6]) + m[7];
        total = lo + hi;
    }
    int c = 0;
    for (int k = 0; k < 8; ++k) {
        if (!((taken >> k) & 1u)) continue;
        pos[c] = k;
        if (nz > 4) value[c] = copysignf(fminf(m[k] / p[k], total), x[k]);
        else        value[c] = x[k];
        ++c;
    }
}

/* test support: how often each position is drawn over all 2^24 uniforms, given the set already drawn */
void oracle_enumerate_draw8(const float x[8], unsigned taken, uint64_t counts[8])
{
    float m[8];
    for (int k = 0; k < 8; ++k) { m[k] = ((taken >> k) & 1u) ? 0.0f : fabsf(x[k]); counts[k] = 0; }
    uint64_t c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    #pragma omp parallel
    {
        uint64_t loc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        #pragma omp for schedule(static)
        for (uint32_t u = 0; u < (1u << 24); ++u) loc[oracle_draw8(m, u24_to_eps(u), taken)] += 1;
        #pragma omp critical
        for (int k = 0; k < 8; ++k) c[k] += loc[k];
    }
    for (int k = 0; k < 8; ++k) counts[k] = c[k];
}

int oracle_prune_4of8_approx(const void *g, int64_t T, int64_t O, int64_t ldg, int dt,
                             uint64_t seed, uint32_t stream_id,
                             void *vals, uint32_t *meta32, void *dense, int64_t ldd)
{
    if (T % 16 || T < 0 || O < 0) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t G = 0; G < T / 16; ++G) {
        for (int64_t o = 0; o < O; ++o) {
            uint32_t md = 0;
            for (int b = 0; b < 2; ++b) {
                int64_t oc = G * 2 + b, t0 = oc * 8;
                float x[8];
                for (int k = 0; k < 8; ++k) x[k] = load_elem(g, dt, (t0 + k) * ldg + o);
                uint32_t u[4];
                oracle_block_u24_quad(seed, stream_id, (uint64_t)oc * (uint64_t)O + (uint64_t)o, u);
                float eps[4];
                for (int d = 0; d < 4; ++d) eps[d] = u24_to_eps(u[d]);
                int pos[4]; float v[4];
                oracle_select_4of8_approx(x, eps, pos, v);
                if (dense) for (int k = 0; k < 8; ++k) store_elem(dense, dt, (t0 + k) * ldd + o, 0.0f);
                for (int s = 0; s < 4; ++s) {
                    float st = store_elem(vals, dt, (G * O + o) * 8 + 4 * b + s, v[s]);
                    md |= (uint32_t)pos[s] << (16 * b + 3 * s);
                    if (dense) store_elem(dense, dt, (t0 + pos[s]) * ldd + o, st);
                }
            }
            meta32[G * O + o] = md;
        }
    }
    return 0;
}

void oracle_nm_decompress_4of8(const void *vals, const uint32_t *meta32, int64_t T, int64_t O, int dt,
                               void *dense, int64_t ldd)
{
    for (int64_t G = 0; G < T / 16; ++G)
        for (int64_t o = 0; o < O; ++o) {
            uint32_t md = meta32[G * O + o];
            for (int b = 0; b < 2; ++b) {
                int64_t t0 = (G * 2 + b) * 8;
                for (int k = 0; k < 8; ++k) {
                    int64_t dst = (t0 + k) * ldd + o;
                    if (dt == DT_F32) ((float *)dense)[dst] = 0.0f; else ((uint16_t *)dense)[dst] = 0;
                }
                for (int s = 0; s < 4; ++s) {
                    int k = (int)((md >> (16 * b + 3 * s)) & 7u);
                    int64_t src = (G * O + o) * 8 + 4 * b + s, dst = (t0 + k) * ldd + o;
                    if (dt == DT_F32) ((float *)dense)[dst] = ((const float *)vals)[src];
                    else ((uint16_t *)dense)[dst] = ((const uint16_t *)vals)[src];
                }
            }
        }
}

/* threads the parallel loops will use (for the benchmark's report) */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
