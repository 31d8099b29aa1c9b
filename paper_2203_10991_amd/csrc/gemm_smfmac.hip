// Update GEMM on CDNA4 sparse MFMA:  dW[O x I] (+)= decompress(vals, meta)^T h   (eq. (3)).
//
// Instruction: v_smfmac_f32_32x32x32_bf16.  "A" is the 4:2-sparse operand (rows = columns o of
// g, i.e. rows of dW), "B" the dense one (h), both reduced over tokens.  Lane layouts, as
// measured on gfx950 (l = lane):
//   A  lane holds 8 kept values of row (l%32) for the 16 tokens  16*(l/32) .. +15  of the
//      32-token step, quad by quad; the 16-bit index word (2 bits per kept value) is exactly one
//      `meta` word of the group format and the 8 values are one 16-byte `vals` fragment.
//   B  lane holds column (l%32); slots 0-7 = tokens 8*(l/32) .. +7, slots 8-15 = tokens
//      16 + 8*(l/32) .. +7.  h is token-major in memory, so the tile is staged in LDS as
//      [token][column] and read with ds_read_b64_tr_b16 (a 4-token x 16-column transpose per
//      16 lanes).
//   D  reg r of lane l = row 8*(r/4) + 4*(l/32) + r%4, column l%32.
//
// Workgroup = WM x WN waves (4: one per SIMD, or 8: two per SIMD), each owning AB x BB accumulator
// blocks of 32x32 in accumulation registers.  The reduction axis advances in stages of 32 tokens (one
// MFMA step).  Every operand byte of a stage -- the h tile, the `vals` fragments and the `meta` words
// of the tile's rows -- is brought from global memory by direct global->LDS loads, once per workgroup
// (the per-CU vector-memory path, 64 B/clk, is the scarce resource: loading the sparse operand per
// wave would fetch it once per wave column).  Six stages rotate through LDS, one barrier per stage; the
// operand registers are double-buffered so that LDS reads of the next stage run under the MFMAs of the
// current one.  Split-K over blockIdx.z writes binary32 partials that a second kernel sums in a
// fixed order (deterministic; no atomics).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <type_traits>
#include <utility>

#include "nm_internal.h"
#include "smfmac_common.h"
#include "gemm_plan.h"

namespace nm {

constexpr int KT = 32;            // tokens per LDS stage (one 32-token MFMA step, two 16-token groups)
constexpr int NS = 6;             // LDS stages: one being consumed, one landed, four in flight

// LDS image of one stage (all filled by direct loads, 64 consecutive lanes -> consecutive LDS bytes):
//   [0, 64*TN)                h tile, [32 tokens][TN columns] bf16, rows unpadded.  Bank conflicts of the
//                             transposing reads are avoided by a swizzle: 16-byte chunk c of row k sits at
//                             chunk position c ^ (4*(k%4)) (a transposing read touches, per 16 lanes, the
//                             same 32-byte column window of 4 consecutive rows).
//   then                      vals fragments, [2 token groups][TM slots] x 16 bytes, one ds_read_b128 per fragment
//   then                      meta words, [2 token groups][TM rows] x 2 bytes
//                             (both as one share per wave, padded to a whole 64-lane load)
// SHIFTED: the dense operand is a set of row-shifted views of one [rows x cb] matrix (a convolution's im2col matrix
// that is never materialised): column block j of h is x read sh.rows[j] rows further down, h[t][j*cb + c] =
// x[(t + rows[j])*ldh + c].  Only a lane's constant source offset and the descriptor's extent change.
template <int WM, int WN, int AB, int BB, bool SHIFTED = false>
__global__ __launch_bounds__(WM * WN * 64) void update_gemm_smfmac_kernel(
    const uint16_t *__restrict__ vals, const uint16_t *__restrict__ meta, const uint16_t *__restrict__ h, int64_t ldh,
    float *__restrict__ out, int64_t ldo, int64_t slab_stride,       // out + z*slab_stride
    int64_t n_groups, int64_t groups_per_slab, int64_t O, int64_t I, int tiles_m, int tiles_n, int accumulate,
    int64_t o_first, int64_t o_end,          // the launch computes rows [o_first, o_end) of dW; tiles_m counts its M-tiles
    ShiftArg sh)                             // (SHIFTED only)
{
    constexpr int TM = WM * AB * 32, TN = WN * BB * 32;
    constexpr int CPR = TN / 8;                           // 16-byte chunks per h row in LDS
    constexpr int ROWS_PER_DMA = 64 / CPR;                // h rows one wave-wide 16-byte direct load covers
    constexpr int NW = WM * WN;                           // waves: 4 (one per SIMD) or 8 (two per SIMD)
    constexpr int WPG = NW / 2;                           // waves that share one of the stage's 2 token groups
    constexpr int B_ROWS = KT / NW;                       // h rows a wave brings per stage
    constexpr int A_ROWS = TM / WPG;                      // tile rows a wave brings (vals and meta) of its token group
    constexpr int B_DMA = B_ROWS / ROWS_PER_DMA;          // direct loads per wave per stage: h tile
    // Every direct load is issued by all 64 lanes (no divergent code in the main loop): a wave's share of the vals
    // fragments is padded to 64 slots and its share of the meta words to 128; the lanes a short share does not
    // need fetch duplicates into the padding.
    constexpr int A_DMA = A_ROWS >= 64 ? A_ROWS / 64 : 1;     //   vals: 64 rows (16 bytes each) per load
    constexpr int A_LANES = A_ROWS >= 64 ? 64 : A_ROWS;
    constexpr int A_SLOTS = A_ROWS >= 64 ? A_ROWS : 64;       //   16-byte slots per share in LDS
    constexpr int M_DMA = A_ROWS >= 128 ? A_ROWS / 128 : 1;   //   meta: 2 words (4 bytes) per lane
    constexpr int M_LANES = A_ROWS >= 128 ? 64 : A_ROWS / 2;  //   (a sub-dword direct load would still land one dword per lane)
    constexpr int M_SLOTS = A_ROWS >= 128 ? A_ROWS : 128;     //   2-byte slots per share in LDS
    static_assert(NW == 4 || NW == 8, "4 or 8 waves");
    static_assert(B_DMA >= 1 && B_ROWS % 4 == 0 && A_ROWS >= 16, "tile too small for this wave count");
    constexpr int LOADS_PER_STAGE = B_DMA + A_DMA + M_DMA;
    constexpr int A_OFF = 64 * TN, M_OFF = A_OFF + 2 * WPG * A_SLOTS * 16;
    constexpr int STAGE_BYTES = (M_OFF + 2 * WPG * M_SLOTS * 2 + 1023) / 1024 * 1024;
    static_assert(CPR >= 16 && CPR <= 64, "tile width");
    static_assert(NS * STAGE_BYTES <= 160 * 1024, "LDS");
    // separate arrays: one per stage in flight
    __shared__ __attribute__((aligned(1024))) char S0[STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char S1[STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char S2[STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char S3[STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char S4[STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char S5[STAGE_BYTES];
    auto buf = [&](auto u_c) -> char * {
        constexpr int u = decltype(u_c)::value % NS;
        if constexpr (u == 0) return S0;
        else if constexpr (u == 1) return S1;
        else if constexpr (u == 2) return S2;
        else if constexpr (u == 3) return S3;
        else if constexpr (u == 4) return S4;
        else return S5;
    };

    int tm, tn, slab;
    tile_and_slab_of_workgroup(tiles_m, tiles_n, tm, tn, slab);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);       // wave-uniform: keeps LDS bases scalar
    const int wm = wave / WN, wn = wave % WN;
    const int64_t m0 = o_first + (int64_t)tm * TM;       // tile's first row of dW (= column of g)
    const int64_t n0 = (int64_t)tn * TN;                 // tile's first column of h / dW
    const int64_t g_begin = (int64_t)slab * groups_per_slab;
    const int64_t g_end = min(n_groups, g_begin + groups_per_slab);
    out += (int64_t)slab * slab_stride;

    f32x16 acc[AB][BB];
#pragma unroll
    for (int a = 0; a < AB; ++a)
#pragma unroll
        for (int b = 0; b < BB; ++b) acc_zero(acc[a][b]);

    const int n_iters = (int)((g_end - g_begin + 1) / 2);      // stages of 2 token groups; the last may be ragged

    // All global reads go through raw buffer descriptors that are re-based as the kernel advances:
    // a 32-bit per-lane offset is all a load needs, and a load from past the end of the tensor (the
    // token group a ragged last stage lacks) is dropped by the bounds check instead of faulting.
    // Split-K slabs are whole stages except the last, so a ragged stage only occurs at the tensor's end.
    auto rsrc = [](const void *base, int64_t bytes) {
        const uint32_t n = bytes <= 0 ? 0u : (bytes > 0xffffffffll ? 0xffffffffu : (uint32_t)bytes);
        return __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)n, 0x00020000);
    };
    const int64_t T = n_groups * 16;

    // per-lane source offsets (bytes, relative to the stage).  Rows >= O and columns >= I are clamped
    // to the last valid ones: their products land in outputs that are never stored.
    const int wgrp = wave / WPG, wsub = wave % WPG;          // this wave's token group of the stage, and its share of the rows
    uint32_t a_src[A_DMA], m_src[M_DMA];
#pragma unroll
    for (int d = 0; d < A_DMA; ++d) {
        // LDS slot q of a token group holds tile row  slot_row(q): inside each wave-row block of AB*32 rows, the 32 rows
        // that feed accumulator block a (rows a, AB+a, 2AB+a, ...) are stored next to each other
        const int q = wsub * A_ROWS + 64 * d + (lane % A_LANES);
        const int row = (q / (AB * 32)) * (AB * 32) + AB * (q % 32) + (q % (AB * 32)) / 32;
        a_src[d] = (uint32_t)(wgrp * O + min(m0 + row, O - 1)) * 16u;
    }
#pragma unroll
    for (int d = 0; d < M_DMA; ++d)
        m_src[d] = (uint32_t)(wgrp * O + min(m0 + wsub * A_ROWS + 128 * d + 2 * (lane % M_LANES), O - 2)) * 2u;
    // h: direct load d of this wave fills rows  wave*B_ROWS + d*ROWS_PER_DMA + lane/CPR  at chunk position
    // lane%CPR, i.e. it must fetch global chunk  (lane%CPR) ^ 4*(row%4).
    constexpr int PHASES = ROWS_PER_DMA >= 4 ? 1 : 4 / ROWS_PER_DMA;
    uint32_t b_src[PHASES];
    const int dma_row = lane / CPR, dma_pos = lane % CPR;
#pragma unroll
    for (int ph = 0; ph < PHASES; ++ph) {
        const int row_mod4 = (ph * ROWS_PER_DMA + dma_row) & 3;
        const int64_t col = min(n0 + 8 * (dma_pos ^ (4 * row_mod4)), I - 8);
        if constexpr (SHIFTED) {
            const int j = (int)(col / sh.cb);             // (a 16-byte chunk never straddles two views: cb % 8 == 0)
            b_src[ph] = (uint32_t)(((int64_t)(wave * B_ROWS + dma_row + sh.rows[j] + sh.margin) * ldh + (col - (int64_t)j * sh.cb)) * 2);
        } else
        b_src[ph] = (uint32_t)(((int64_t)(wave * B_ROWS + dma_row) * ldh + col) * 2);
    }
    const uint32_t b_row_step = (uint32_t)(ROWS_PER_DMA * ldh * 2);

    // Buffer descriptors are re-based once per trip of NS stages (to the trip's first stage, with the exact
    // number of bytes left in the tensor as the bound); a stage inside or ahead of the trip is reached through
    // the per-lane offset.  U = stage number relative to the descriptors' stage, at most 2*NS-1.
    __amdgpu_buffer_rsrc_t rh, rv, rm;
    auto rebase = [&](int it) {
        const int64_t Gs = g_begin + (int64_t)it * 2, t0 = Gs * 16;
        if constexpr (SHIFTED)       // rows -margin .. T+margin-1 of x are readable; offsets are relative to row t0 - margin
            rh = rsrc((const char *)h + (t0 - sh.margin) * ldh * 2, ((T - t0 - 1 + 2 * (int64_t)sh.margin) * ldh + sh.cb) * 2);
        else
        rh = rsrc((const char *)h + t0 * ldh * 2, ((T - t0 - 1) * ldh + I) * 2);
        rv = rsrc((const char *)vals + Gs * O * 16, (n_groups - Gs) * O * 16);
        rm = rsrc((const char *)meta + Gs * O * 2, (n_groups - Gs) * O * 2);
    };
    const uint32_t h_stage = (uint32_t)(KT * ldh * 2), v_stage = (uint32_t)(2 * O * 16), m_stage = (uint32_t)(2 * O * 2);
    // direct load number K (of LOADS_PER_STAGE) of the stage U stages past the descriptors' one
    auto fetch_one = [&](auto u_c, auto k_c, char *stage) {
        constexpr uint32_t U = decltype(u_c)::value;
        constexpr int K = decltype(k_c)::value;
        if constexpr (K < B_DMA)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rh, (lptr_t)(stage + (wave * B_ROWS + K * ROWS_PER_DMA) * (TN * 2)), 16,
                                                     (int)(b_src[K % PHASES] + (uint32_t)K * b_row_step + U * h_stage), 0, 0, 0);
        else if constexpr (K < B_DMA + A_DMA)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rv, (lptr_t)(stage + A_OFF + (wave * A_SLOTS + 64 * (K - B_DMA)) * 16), 16,
                                                     (int)(a_src[K - B_DMA] + U * v_stage), 0, 0, 0);
        else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rm, (lptr_t)(stage + M_OFF + wave * M_SLOTS * 2 + (K - B_DMA - A_DMA) * 256), 4,
                                                     (int)(m_src[K - B_DMA - A_DMA] + U * m_stage), 0, 0, 0);
    };
    auto fetch = [&](auto u_c, char *stage) {
        static_for<LOADS_PER_STAGE>([&](auto k_c) { fetch_one(u_c, k_c, stage); });
    };
    // first stage (relative to the slab) in which this wave's token group lies past the end of the tensor
    const int first_missing = (int)min((int64_t)0x7fffffff, (n_groups - g_begin - wgrp + 1) / 2);
    // "stage `it` has landed" while the loads of the IN_FLIGHT stages fetched after it may still be on
    // their way ...
    auto stage_ready = [&](auto in_flight_c, int it, char *stage) {
        wait_vmcnt<decltype(in_flight_c)::value * LOADS_PER_STAGE>();
        // A direct load whose source lies past the end of the tensor leaves its LDS bytes untouched.
        // Each wave brought a share of one token group of the stage (h rows, vals fragments, meta
        // words): if that group does not exist, the wave clears what it would have brought.
        if (it >= first_missing) {
            const uint4 z = make_uint4(0, 0, 0, 0);
            for (int c = lane; c < B_ROWS * CPR; c += 64) *(uint4 *)(stage + wave * B_ROWS * (TN * 2) + c * 16) = z;
            for (int c = lane; c < A_SLOTS; c += 64) *(uint4 *)(stage + A_OFF + (wave * A_SLOTS + c) * 16) = z;
            for (int c = lane; c < M_SLOTS / 8; c += 64) *(uint4 *)(stage + M_OFF + wave * M_SLOTS * 2 + c * 16) = z;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        // ... and every other wave's part of it too.  A bare barrier: __syncthreads() would add a
        // workgroup release fence, which the compiler implements by draining every direct-to-LDS
        // load in flight (those of the later stages included).
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };

    // lane's LDS read addresses inside a stage
    const int li = lane & 15, q4 = lane >> 4, kg = lane >> 5;
    const int rd_row = (8 * (q4 >> 1) + (li >> 2)) * (TN * 2);     // h: + (16*(j>>1) + 4*(j&1)) rows for read j of a fragment
    uint32_t rd_b[BB];
#pragma unroll
    for (int b = 0; b < BB; ++b)
        rd_b[b] = (uint32_t)(rd_row + (4 * (((wn * BB + b)) ^ (li >> 2)) + 2 * (q4 & 1) + ((li & 3) >> 1)) * 16 + (li & 1) * 8);
    // slot q (row r) of token group kg sits in the share of wave  kg*WPG + q/A_ROWS  at position  q % A_ROWS
    constexpr int A_BLOCK = (A_ROWS >= 64 ? 32 : 64) * 16;       // bytes between the fragments of consecutive accumulator blocks
    static_assert(A_ROWS % 32 == 0 && (AB * 32) % A_ROWS == 0 || A_ROWS % (AB * 32) == 0, "shares and wave rows nest");
    const int q0 = wm * (AB * 32), r0 = q0 + AB * (lane & 31);
    const uint32_t rd_a = (uint32_t)(A_OFF + ((kg * WPG + q0 / A_ROWS) * A_SLOTS + q0 % A_ROWS + (lane & 31)) * 16);   // + a*A_BLOCK
    const uint32_t rd_m = (uint32_t)(M_OFF + ((kg * WPG + r0 / A_ROWS) * M_SLOTS + r0 % A_ROWS) * 2);                   // AB consecutive words

    // Operand registers: two sets.  While the MFMAs of a stage read one set, the LDS reads of the next
    // stage fill the other, so the fragment pipeline never drains at a stage boundary.
    static_assert(AB == 2 || AB == 4, "AB is 2 or 4");
    Frag8 af[2][AB];
    u32x2 ix2[2]; uint32_t ix1[2];          // index words as read, AB consecutive 16-bit words: the one that matches AB is used
    Frag16 bf[2][BB];
    constexpr int NR = AB + 1 + 4 * BB;     // LDS reads of one stage per wave
    constexpr int NM = AB * BB;             // MFMAs of one stage per wave
    static_assert(NR <= 15, "lgkmcnt is a 4-bit counter");
    // read number r of a stage, in issue order: AB sparse fragments, the index words, 4 reads per h fragment
    auto lds_read = [&](auto set_c, auto r_c, char *stage) {
        constexpr int set = decltype(set_c)::value, r = decltype(r_c)::value, R = TN * 2;
        const uint32_t base = (uint32_t)(uintptr_t)(lptr_t)stage;
        if constexpr (r < AB) af[set][r].u4 = lds_read_b128<r * A_BLOCK>(base + rd_a);
        else if constexpr (r == AB) {
            if constexpr (AB == 4) ix2[set] = lds_read_b64<0>(base + rd_m);
            else                   ix1[set] = lds_read_b32<0>(base + rd_m);
        } else {
            constexpr int j = r - AB - 1, b = j / 4, qd = j % 4;
            bf[set][b].q[qd] = lds_read_tr16<(16 * (qd >> 1) + 4 * (qd & 1)) * R>(base + rd_b[b]);
        }
    };
    // One stage: its operands are in (or on their way into) register set SET; its MFMAs are
    // interleaved with the LDS reads of the following stage (from `next`) into the other set.
    // The direct loads of the stage FU stages ahead (into `far`) are spread over the MFMAs as well: issued in one
    // burst they fill the CU's vector-memory queue, and the waves stall on them instead of feeding the matrix pipeline.
    auto consume = [&](auto set_c, char *next, auto fu_c, char *far) {
        constexpr int set = decltype(set_c)::value;
        constexpr int NL = LOADS_PER_STAGE;
        // every read of this stage was issued during the previous stage.  The wait names the index-word
        // registers as an operand, so that the compiler cannot move their (its own) uses above it.
        if constexpr (AB == 4) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(ix2[set]));
        else                   asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(ix1[set]));
        static_for<NM>([&](auto m_c) {
            constexpr int m = decltype(m_c)::value, b = m / AB, a = m % AB;
            uint32_t idx;
            if constexpr (AB == 4) idx = ix2[set][a / 2];
            else                   idx = ix1[set];
            smfmac_32x32x32<-1, (a & 1)>(acc[a][b], af[set][a].v, bf[set][b].v, idx);
            static_for<NR>([&](auto r_c) {
                constexpr int r = decltype(r_c)::value;
                if constexpr (r >= m * NR / NM && r < (m + 1) * NR / NM) lds_read(std::integral_constant<int, 1 - set>{}, r_c, next);
            });
            static_for<NL>([&](auto k_c) {
                constexpr int k = decltype(k_c)::value;
                if constexpr (k >= m * NL / NM && k < (m + 1) * NL / NM) fetch_one(fu_c, k_c, far);
            });
        });
    };

    // Six LDS stages rotating.  During stage j: stage j+1 has landed (its readiness barrier opens the
    // slot), the loads of stages j+2 .. j+4 are in flight and those of stage j+5 are issued into the
    // buffer that stage j-1 occupied -- every wave finished reading it before it arrived at this slot's
    // barrier.  A load therefore has four stages of MFMA work (about two thousand cycles) to land.
    // Straight-line loop body, six stages per trip.  Stages past the end of the tensor hold zeros
    // (dropped loads, cleared shares), so the stage count is padded to a multiple of six with
    // all-zero stages and the fetches and reads that run ahead of the last stage need no guard.
    // (Split-K slabs other than the last hold a multiple of six stages: see make_plan.)
    const int n_trips = (n_iters + NS - 1) / NS;
    if (n_trips > 0) {
        rebase(0);
        static_for<NS - 1>([&](auto u_c) { fetch(u_c, buf(u_c)); });
        stage_ready(std::integral_constant<int, NS - 2>{}, 0, S0);
        static_for<NR>([&](auto r_c) { lds_read(std::integral_constant<int, 0>{}, r_c, S0); });
    }
    for (int tr = 0; tr < n_trips; ++tr) {
        const int it = NS * tr;
        rebase(it);
        static_for<NS>([&](auto u_c) {
            constexpr int u = decltype(u_c)::value;
            stage_ready(std::integral_constant<int, NS - 3>{}, it + u + 1, buf(std::integral_constant<int, u + 1>{}));
            consume(std::integral_constant<int, u % 2>{}, buf(std::integral_constant<int, u + 1>{}),
                    std::integral_constant<int, u + NS - 1>{}, buf(std::integral_constant<int, u + NS - 1>{}));
        });
    }

    // ---- epilogue.  The matrix pipeline may still be writing the last accumulators, and the
    // compiler cannot see MFMAs inside asm statements: idle for longer than an 8-pass
    // instruction before the first read of an accumulation register.
    // (The reads issued ahead for the stage after the last are drained first: their destination registers are dead.)
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
    for (int a = 0; a < AB; ++a)
#pragma unroll
        for (int b = 0; b < BB; ++b) acc_settled(acc[a][b]);
    __builtin_amdgcn_sched_barrier(0);
    const int64_t o0 = m0 + wm * (AB * 32);
#pragma unroll
    for (int a = 0; a < AB; ++a)
#pragma unroll
        for (int b = 0; b < BB; ++b) {
            const int64_t col = n0 + wn * (BB * 32) + b * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = o0 + AB * (8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) + a;   // block a holds rows a, AB+a, ...
                if (row < o_end && col < I) {
                    float *p = out + row * ldo + col;
                    if (accumulate) *p = *p + acc[a][b][r];
                    else store_acc(p, acc[a][b][r]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);       // one block at a time: keeps the address arithmetic of 16 stores, not of all, live
        }
}

// ------------------------------------------------------------------------------------
// 384 x 256 tile.  What bounds the 256 x 256 kernel on large problems is the path from the L2s to the
// CUs (0.8 KB of operands per token and tile); a tile that is 1.5 times taller needs 21 % fewer bytes
// per product.  8 waves as 2 x 4, wave tile 192 x 64 = 6 x 2 accumulator blocks (192 accumulation
// registers), which leaves 64 ordinary registers per wave: the operand registers are single and are
// refilled in place -- a fragment of the next stage is read into the registers of the same fragment of
// the current stage right after the last MFMA that uses them.  MFMA order inside a stage: the six row
// blocks against column block 0, then against column block 1; so column fragment 0 is refilled after
// MFMA 6, row fragment a after MFMA 7+a, column fragment 1 after MFMA 12.
//
// Rows of a wave's 192-row block are interleaved so that the index words a lane needs are adjacent in
// the natural `meta` order: accumulator block a holds rows 6m + a of the wave's 192 rows (m = row inside
// the block), so a lane's six index words are 12 consecutive bytes.
// LDS image of a stage: h tile [32][256] bf16 (swizzled as above) | vals [2 groups][384 slots] x 16 B
// (slot 192*wm + 32*a + m) | meta [2 groups][384 rows] x 2 B; five stages rotate.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void update_gemm_smfmac_tall_kernel(
    const uint16_t *__restrict__ vals, const uint16_t *__restrict__ meta, const uint16_t *__restrict__ h, int64_t ldh,
    float *__restrict__ out, int64_t ldo, int64_t slab_stride, int64_t n_groups, int64_t groups_per_slab,
    int64_t O, int64_t I, int tiles_m, int tiles_n, int accumulate, int64_t o_first, int64_t o_end)
{
    constexpr int WN = 4, AB = 6, BB = 2, TM = 384, TN = 256, TNS = 5;
    constexpr int A_OFF = 64 * TN, M_OFF = A_OFF + 2 * TM * 16, STAGE = (M_OFF + 2 * TM * 2 + 1023) / 1024 * 1024;
    constexpr int LPS = 5;                                   // direct loads per wave and stage: 2 h, 2 vals, 1 meta
    static_assert(TNS * STAGE <= 160 * 1024, "LDS");
    __shared__ __attribute__((aligned(1024))) char S[TNS * STAGE];

    int tm, tn;
    tile_of_workgroup((int)blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int64_t m0 = o_first + (int64_t)tm * TM, n0 = (int64_t)tn * TN;
    const int64_t g_begin = (int64_t)blockIdx.z * groups_per_slab;
    const int64_t g_end = min(n_groups, g_begin + groups_per_slab);
    out += (int64_t)blockIdx.z * slab_stride;

    // accumulator blocks of rows a < 4 in accumulation registers (128), a = 4, 5 in ordinary ones (64)
    f32x16 acc[AB][BB];
    static_for<AB>([&](auto a_c) {
        constexpr int a = decltype(a_c)::value;
        static_for<BB>([&](auto b_c) { acc_zero<(a >= 4)>(acc[a][decltype(b_c)::value]); });
    });

    const int n_iters = (int)((g_end - g_begin + 1) / 2);      // stages of 2 token groups; the last may be ragged
    const int n_trips = (n_iters + TNS - 1) / TNS;

    // tile row held by slot q of a token group (see above)
    auto slot_row = [](int q) {
        const int blk = q / 192, r = q % 192, a = r / 32, m = r % 32;
        return blk * 192 + 6 * m + a;
    };
    // ---- direct loads.  Wave w brings, of token group w/4 of the stage and with ws = w%4: 4 rows of h (2 loads of
    // 64 lanes), vals slots [96 ws, 96 ws + 96) (one load of 64 lanes and one of the low 32 lanes), meta rows
    // [96 ws, 96 ws + 96) (one load of the low 48 lanes, two words each): every slot and row of the tile once.  The
    // lane-masked loads still count for every wave: vmcnt advances by LPS = 5 per stage whatever the mask, which is
    // what the waits in stage_ready assume.  Per-lane byte offsets inside a stage; the stage itself is reached through
    // the scalar offset, which the bounds check does not cover: a load for a token group past the end of the tensor is
    // switched off through the descriptor's size instead.
    const int wgrp = wave / 4, ws = wave % 4;
    uint32_t b_src[2], a_src[2], m_src;
    {
        constexpr int CPR = TN / 8;                          // 32 chunks of 16 bytes per h row
        const int dma_row = lane / CPR, dma_pos = lane % CPR;
#pragma unroll
        for (int ph = 0; ph < 2; ++ph) {                     // load d covers rows 4*wave + 2*d + dma_row
            const int row_mod4 = (2 * ph + dma_row) & 3;
            const int64_t col = min(n0 + 8 * (dma_pos ^ (4 * row_mod4)), I - 8);
            b_src[ph] = (uint32_t)(((int64_t)(wave * 4 + 2 * ph + dma_row) * ldh + col) * 2);
        }
        // vals: slots [96*ws, 96*ws+96) as one 64-lane and one 32-lane load; meta: rows [96*ws, 96*ws+96) as 48 lanes
#pragma unroll
        for (int d = 0; d < 2; ++d)
            a_src[d] = (uint32_t)(wgrp * O + min(m0 + slot_row(96 * ws + 64 * d + (d ? (lane & 31) : lane)), O - 1)) * 16u;
        m_src = (uint32_t)(wgrp * O + min(m0 + 96 * ws + 2 * (lane % 48), O - 2)) * 2u;
    }
    const bool lane_lt32 = lane < 32, lane_lt48 = lane < 48;
    const uint32_t h_stage = (uint32_t)(KT * ldh * 2), v_stage = (uint32_t)(2 * O * 16), m_stage = (uint32_t)(2 * O * 2);
    const int first_missing = (int)min((int64_t)0x7fffffff, (n_groups - g_begin - wgrp + 1) / 2);
    const char *hp = nullptr, *vp = nullptr, *mp = nullptr;   // the tensors at the first stage of the current trip
    int trip_first = 0;
    auto rebase = [&](int it) {
        const int64_t Gs = g_begin + (int64_t)it * 2;
        hp = (const char *)h + Gs * 16 * ldh * 2;
        vp = (const char *)vals + Gs * O * 16;
        mp = (const char *)meta + Gs * O * 2;
        trip_first = it;
    };
    // load K of the stage U stages past the trip's first one, into stage buffer BUF
    auto fetch_one = [&](auto u_c, auto k_c, auto buf_c) {
        constexpr uint32_t U = decltype(u_c)::value;
        constexpr int K = decltype(k_c)::value, BUF = decltype(buf_c)::value % TNS;
        const int size = trip_first + (int)U < first_missing ? 0x7fffffff : 0;        // 0: every lane out of range, nothing is loaded
        char *stage = S + BUF * STAGE;
        if constexpr (K < 2)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(__builtin_amdgcn_make_buffer_rsrc((void *)hp, 0, size, 0x00020000),
                                                     (lptr_t)(stage + (wave * 4 + 2 * K) * (TN * 2)), 16, (int)b_src[K],
                                                     (int)(U * h_stage), 0, 0);
        else if constexpr (K == 2)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(__builtin_amdgcn_make_buffer_rsrc((void *)vp, 0, size, 0x00020000),
                                                     (lptr_t)(stage + A_OFF + (wgrp * TM + 96 * ws) * 16), 16,
                                                     (int)a_src[0], (int)(U * v_stage), 0, 0);
        else if constexpr (K == 3) {
            if (lane_lt32)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(__builtin_amdgcn_make_buffer_rsrc((void *)vp, 0, size, 0x00020000),
                                                         (lptr_t)(stage + A_OFF + (wgrp * TM + 96 * ws + 64) * 16), 16,
                                                         (int)a_src[1], (int)(U * v_stage), 0, 0);
        } else {
            if (lane_lt48)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(__builtin_amdgcn_make_buffer_rsrc((void *)mp, 0, size, 0x00020000),
                                                         (lptr_t)(stage + M_OFF + (wgrp * TM + 96 * ws) * 2), 4, (int)m_src,
                                                         (int)(U * m_stage), 0, 0);
        }
    };
    // "stage `it` has landed" with the loads of IN_FLIGHT later stages still on their way; a wave whose token
    // group lies past the end of the tensor clears what it would have brought (its loads were switched off)
    auto stage_ready = [&](auto in_flight_c, int it, auto buf_c) {
        constexpr int BUF = decltype(buf_c)::value % TNS;
        wait_vmcnt<decltype(in_flight_c)::value * LPS>();
        if (it >= first_missing) {
            // zero kept values make the group's products zero whatever the index words left in the buffer are; the h
            // rows are cleared too (a buffer no load has reached yet may hold NaN patterns).  Everything the branch
            // needs is made inside it: nothing of it occupies a register on the common path.
            char *stage = S + BUF * STAGE;
            uint32_t zero, ln;
            asm volatile("v_mov_b32 %0, 0\n\tv_mbcnt_lo_u32_b32 %1, -1, 0\n\tv_mbcnt_hi_u32_b32 %1, -1, %1" : "=v"(zero), "=v"(ln));
            const uint4 z = make_uint4(zero, zero, zero, zero);
            *(uint4 *)(stage + A_OFF + (wgrp * TM + 96 * ws + ln) * 16) = z;
            if (ln < 32) *(uint4 *)(stage + A_OFF + (wgrp * TM + 96 * ws + 64 + ln) * 16) = z;
            *(uint4 *)(stage + wave * 4 * (TN * 2) + ln * 16) = z;
            *(uint4 *)(stage + wave * 4 * (TN * 2) + 1024 + ln * 16) = z;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- LDS read addresses of the stage being read; they advance by one stage per slot
    const int li = lane & 15, q4 = lane >> 4, kg = lane >> 5, m = lane & 31;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)S;
    uint32_t cur_a = lds0 + (uint32_t)(A_OFF + (kg * TM + wm * 192 + m) * 16);                 // + 32*a*16
    uint32_t cur_m = lds0 + (uint32_t)(M_OFF + (kg * TM + wm * 192 + 6 * m) * 2);              // 6 consecutive words (three reads)
    // column block b of wave wn is block b*4 + wn of the tile: the swizzle only touches the low two bits of that
    // number, so the two blocks of a wave are a constant 256 bytes apart in every row
    uint32_t cur_b = lds0 + (uint32_t)((8 * (q4 >> 1) + (li >> 2)) * (TN * 2) +
                                       (4 * (wn ^ (li >> 2)) + 2 * (q4 & 1) + ((li & 3) >> 1)) * 16 + (li & 1) * 8);
    // (asm: the compiler would otherwise keep one copy of every address per stage buffer)
    auto advance = [&](int bytes) {
        asm volatile("v_add_u32 %0, %3, %0\n\tv_add_u32 %1, %3, %1\n\tv_add_u32 %2, %3, %2" : "+v"(cur_a), "+v"(cur_m), "+v"(cur_b) : "s"(bytes));
    };

    Frag8 af[AB];
    Frag16 bf[BB];
    uint32_t ix[3] = {0, 0, 0};                              // index words of blocks (0,1), (2,3), (4,5): low and high half
#pragma unroll
    for (int a = 0; a < AB; ++a) af[a].u4 = u32x4{0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < BB; ++b)
#pragma unroll
        for (int j = 0; j < 4; ++j) bf[b].q[j] = s16x4{0, 0, 0, 0};
    auto read_a = [&](auto a_c) { constexpr int a = decltype(a_c)::value; lds_refill_b128<32 * a * 16>(af[a].u4, cur_a); };
    auto read_ix = [&](auto j_c) {
        constexpr int j = decltype(j_c)::value;
        lds_refill_b32<4 * j>(ix[j], cur_m);
    };
    auto read_b = [&](auto b_c) {
        constexpr int b = decltype(b_c)::value, R = TN * 2;
        lds_refill_tr16<0 * R + 256 * b>(bf[b].q[0], cur_b);
        lds_refill_tr16<4 * R + 256 * b>(bf[b].q[1], cur_b);
        lds_refill_tr16<16 * R + 256 * b>(bf[b].q[2], cur_b);
        lds_refill_tr16<20 * R + 256 * b>(bf[b].q[3], cur_b);
    };
    // LDS reads of one stage, in issue order (the waits below count on it):
    //   B0 (4 reads) | A0 | A1, ix0 | A2 | A3, ix1 | A4 | A5, ix2, B1 (4)
    // One stage of MFMAs.  Before MFMA number n (1..12) the reads issued after the ones it needs may still be
    // outstanding: that count is the wait.  After it: the refill of what it freed, and a share of the direct loads.
    auto mfma = [&](auto a_c, auto b_c) {
        constexpr int a = decltype(a_c)::value, b = decltype(b_c)::value;
        smfmac_32x32x32<-1, (a & 1), (a >= 4)>(acc[a][b], af[a].v, bf[b].v, ix[a / 2]);
    };
    auto lgkm_wait = [&](auto n_c, auto) { asm volatile("s_waitcnt lgkmcnt(%0)" : : "n"(decltype(n_c)::value)); };
    using I0 = std::integral_constant<int, 0>; using I1 = std::integral_constant<int, 1>; using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>; using I4 = std::integral_constant<int, 4>; using I5 = std::integral_constant<int, 5>;
    auto consume = [&](auto fu_c, auto fbuf_c) {
        lgkm_wait(std::integral_constant<int, 10>{}, I0{}); mfma(I0{}, I0{});
        fetch_one(fu_c, I0{}, fbuf_c);
        mfma(I1{}, I0{});
        lgkm_wait(std::integral_constant<int, 7>{}, I2{});  mfma(I2{}, I0{});
        fetch_one(fu_c, I1{}, fbuf_c);
        mfma(I3{}, I0{});
        lgkm_wait(std::integral_constant<int, 4>{}, I4{});  mfma(I4{}, I0{});     // (ix2 is the last read before B1)
        fetch_one(fu_c, I2{}, fbuf_c);
        mfma(I5{}, I0{});
        read_b(I0{});
        asm volatile("s_waitcnt lgkmcnt(4)");
        mfma(I0{}, I1{}); read_a(I0{});
        mfma(I1{}, I1{}); read_a(I1{}); read_ix(I0{});
        fetch_one(fu_c, I3{}, fbuf_c);
        mfma(I2{}, I1{}); read_a(I2{});
        mfma(I3{}, I1{}); read_a(I3{}); read_ix(I1{});
        fetch_one(fu_c, I4{}, fbuf_c);
        mfma(I4{}, I1{}); read_a(I4{});
        mfma(I5{}, I1{}); read_a(I5{}); read_ix(I2{}); read_b(I1{});
    };
    auto read_all = [&]() {
        read_b(I0{}); read_a(I0{}); read_a(I1{}); read_ix(I0{}); read_a(I2{}); read_a(I3{}); read_ix(I1{}); read_a(I4{});
        read_a(I5{}); read_ix(I2{}); read_b(I1{});
    };

    // Five LDS stages.  Slot j: stage j's operands are in (or on their way into) registers, read during slot j-1;
    // stage j+1 has landed (the barrier that opens the slot) and is read during the slot; the loads of stages j+2 and
    // j+3 are in flight, those of stage j+4 are issued into the buffer stage j-1 occupied (every wave finished reading
    // it before it arrived at this slot's barrier).  Stages past the end of the tensor hold zeros, so the stage count
    // is padded to a multiple of five and nothing that runs ahead needs a guard.
    if (n_trips > 0) {
        rebase(0);
        static_for<TNS - 1>([&](auto u_c) { static_for<LPS>([&](auto k_c) { fetch_one(u_c, k_c, u_c); }); });
        stage_ready(std::integral_constant<int, TNS - 2>{}, 0, I0{});
        read_all();
        advance(STAGE);
    }
    for (int tr = 0; tr < n_trips; ++tr) {
        const int it = TNS * tr;
        rebase(it);
        static_for<TNS>([&](auto u_c) {
            constexpr int u = decltype(u_c)::value;
            stage_ready(std::integral_constant<int, TNS - 3>{}, it + u + 1, std::integral_constant<int, u + 1>{});
            consume(std::integral_constant<int, u + TNS - 1>{}, std::integral_constant<int, u + TNS - 1>{});
            advance(u == TNS - 2 ? -(TNS - 1) * STAGE : STAGE);       // the reads of the next slot take the stage after
        });
    }

    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
    static_for<AB>([&](auto a_c) {
        constexpr int a = decltype(a_c)::value;
#pragma unroll
        for (int b = 0; b < BB; ++b) acc_settled<(a >= 4)>(acc[a][b]);
    });
    __builtin_amdgcn_sched_barrier(0);
    static_for<AB>([&](auto a_c) {
        constexpr int a = decltype(a_c)::value;
#pragma unroll
        for (int b = 0; b < BB; ++b) {
            const int64_t col = n0 + (b * 4 + wn) * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int mr = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);               // row inside the accumulator block
                const int64_t row = m0 + wm * 192 + 6 * mr + a;
                if (row < o_end && col < I) {
                    float *p = out + row * ldo + col;
                    if (accumulate) *p = *p + acc[a][b][r];
                    else store_acc<(a >= 4)>(p, acc[a][b][r]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);       // one block at a time
        }
    });
}

// out[o][i] = (accumulate ? out : 0) + alpha * sum_z part[z][o][i].  R threads share one float4 of the output
// (R = 1 for a few slabs, 8 for many): thread r sums the slabs z = r, r+R, ... in ascending order, then the R partial
// sums are combined in a fixed tree (neighbours at distance 1, 2, 4): the order of the additions depends on the slab
// count only, never on timing.
template <int R>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ part, int slabs, int64_t slab_stride,
                                                           float *__restrict__ out, int64_t ldo, int64_t O, int64_t I, int accumulate,
                                                           AlphaArg al)
{
    const float alpha = alpha_of(al);
    const int64_t n4 = O * (I / 4);
    const int r = threadIdx.x % R;
    const int64_t idx = (int64_t)blockIdx.x * (256 / R) + threadIdx.x / R;
    const bool valid = idx < n4;
    const int64_t o = valid ? idx / (I / 4) : 0, i = valid ? (idx % (I / 4)) * 4 : 0;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (valid)
        for (int z = r; z < slabs; z += R) {
            const float4 v = *(const float4 *)(part + (int64_t)z * slab_stride + o * I + i);
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
#pragma unroll
    for (int d = 1; d < R; d <<= 1) {
        s.x += __shfl_xor(s.x, d); s.y += __shfl_xor(s.y, d); s.z += __shfl_xor(s.z, d); s.w += __shfl_xor(s.w, d);
    }
    if (!valid || r != 0) return;
    s.x *= alpha; s.y *= alpha; s.z *= alpha; s.w *= alpha;
    if (accumulate) {
        const float4 d = *(const float4 *)(out + o * ldo + i);
        s.x += d.x; s.y += d.y; s.z += d.z; s.w += d.w;
    }
    *(float4 *)(out + o * ldo + i) = s;
}

// dW = (accumulate ? dW : 0) + alpha * sum over the slabs of [slabs][O][I] partial sums (row stride I), in slab order
hipError_t launch_splitk_reduce(const float *part, int slabs, float *dW, int64_t lddw, int64_t O, int64_t I,
                                int accumulate, AlphaArg alpha, hipStream_t st)
{
    const int64_t n4 = O * (I / 4);
    if (slabs >= 12)
        hipLaunchKernelGGL(splitk_reduce_kernel<8>, dim3((unsigned)((n4 + 31) / 32)), dim3(256), 0, st, part, slabs, O * I,
                           dW, lddw, O, I, accumulate, alpha);
    else
        hipLaunchKernelGGL(splitk_reduce_kernel<1>, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, part, slabs, O * I,
                           dW, lddw, O, I, accumulate, alpha);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// host side: tile shape and split-K plan (pure function of the problem size)
// ------------------------------------------------------------------------------------
// tall_rows: rows [0, tall_rows) of dW are computed by the 384 x 256 kernel (tall_tiles_m tile rows), the rest by the
// kernel of `shape` (tiles_m tile rows); 0 = that kernel alone.
struct Plan { int shape; int tm, tn; int tiles_m, tiles_n; int slabs; int64_t groups_per_slab; int64_t tall_rows; int tall_tiles_m; };

// shifted: the dense operand is row-shifted views of one matrix (it stays in the caches: few-row problems are then
// bound by the tile's own work, and the 64 x 256 tile wastes none of it; streamed from HBM, as a materialised
// operand is, the 128 x 128 tile measures faster)
static Plan make_plan(int64_t T, int64_t O, int64_t I, bool shifted = false)
{
    Plan p;
    const int64_t groups = T / 16;
    const int CUS = 256;
    p.tall_rows = 0; p.tall_tiles_m = 0;
    // shape 0: 256x256 (8 waves), shape 1: 128x128 (4 waves, two workgroups fit a CU), shape 2: 64x256 (4 waves, one per CU),
    // shape 3: 256x128 (8 waves, one per CU)
    bool small = false;
    if ((O + 255) / 256 * ((I + 255) / 256) >= CUS) {
        p.shape = 0; p.tm = 256; p.tn = 256;
        // Large problems: rows split between the 384 x 256 kernel (21 % fewer operand bytes per product, ~10 % faster
        // per product, a round of its tiles 1.34 times as long) and the 256 x 256 kernel
        const RowSplit rs = split_rows_tall(O, I, 1.34, !shifted);
        p.tall_tiles_m = rs.tall_tiles_m;
        p.tall_rows = rs.tall_rows;
    }
    else if (shifted && O <= 64 && I > 128) { p.shape = 2; p.tm = 64; p.tn = 256; small = true; }
    else { p.shape = 1; p.tm = 128; p.tn = 128; small = true; }
    p.tiles_m = (int)((O - p.tall_rows + p.tm - 1) / p.tm);
    p.tiles_n = (int)((I + p.tn - 1) / p.tn);
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    // Smaller problems: the reduction axis is cut into slabs until the GPU is filled evenly -- one workgroup on every
    // CU, or two on (nearly) every CU; anything between leaves some CUs with twice the work of the others.  Of the two
    // the cheaper one by a measured cost model: microseconds per 32-token stage of a 128 x 128 tile (0.14 alone on
    // its CU, rising to 0.18 with all CUs busy; 0.32 when two share a CU), never less than one pass over the operands
    // at 4.5 TB/s, plus the second pass over the partial sums.
    // Then the same problem on 256 x 256 tiles, cut into as many slabs as keep it to one workgroup per CU: half the
    // operand bytes per product, more partial sums.  The two are compared with the stage costs measured on operands
    // that are not in any cache, as a training step finds them (128 x 128: 0.19-0.25 us, 0.42 with two on a CU;
    // 256 x 256: 0.44-0.56 us plus 3 us of pipeline fill): the small tile loses more to cold operands than the large.
    // The large tile has to win by 15 %: its plan writes two to three times the partial sums and leaves no CU to a
    // kernel that runs beside it (layers replayed from a graph with parallel branches measure 5 % slower with it
    // where the margin is smaller).
    // Between the two sits a 256 x 128 tile on 8 waves (one workgroup per CU, 102 KB of LDS: 0.30-0.365 us per stage cold, a
    // third fewer operand bytes per product than 128 x 128; the same tile on 4 waves measured 2-9 % slower): it takes the
    // ViT-sized layers (qkv, fc1, fc2) at the same or a little more workspace when predicted 5 % faster.
    auto whole_trips = [](int64_t gps) { gps = (gps + 11) / 12 * 12; return gps < 12 ? (int64_t)12 : gps; };
    int slabs = 1;
    if (small && groups >= 48) {
        const int64_t max_s = std::max<int64_t>(1, groups / 24);               // at least 384 tokens per slab
        auto second_pass = [&](int64_t sl) { return sl > 1 ? 4.0 + (double)(sl + 1) * (double)O * (double)I * 4.0 / 3.5e6 : 0.0; };
        const double stream = (double)T * ((double)I * 2.0 + (double)O * 1.125) / 4.5e6;
        auto cost = [&](int64_t sl, bool cold) {
            const int64_t wgs = tiles * sl, stages = whole_trips((groups + sl - 1) / sl) / 2;
            const double fill = (double)wgs / CUS;
            const double t_stage = cold ? (wgs <= CUS ? 0.19 + 0.06 * fill : 0.42) : (wgs <= CUS ? 0.14 + 0.04 * fill : 0.32);
            const double rounds = wgs <= CUS ? 1.0 : (double)((wgs + 2 * CUS - 1) / (2 * CUS));
            return std::max(rounds * (double)stages * t_stage, stream) + second_pass(sl);
        };
        const int64_t s_one = std::min(max_s, std::max<int64_t>(1, CUS / tiles));
        const int64_t s_two = std::min(max_s, std::max<int64_t>(1, 2 * CUS / tiles));
        slabs = (int)s_one;
        if (p.shape == 1 && tiles * s_two >= 3 * CUS / 2 && cost(s_two, false) < cost(s_one, false)) slabs = (int)s_two;
        if (p.shape == 1) {
            // one workgroup per CU at most on the larger tiles: cost of `tl` tiles cut into as many slabs as fit, at
            // t_lo us per stage up to a `knee` share of the CUs in use, rising linearly to t_hi with all of them
            auto one_per_cu = [&](int64_t tl, double t_lo, double t_hi, double knee, int64_t &sl) {
                sl = std::min(max_s, std::max<int64_t>(1, CUS / tl));
                const int64_t wgs = tl * sl, stages = whole_trips((groups + sl - 1) / sl) / 2;
                const double rounds = (double)((wgs + CUS - 1) / CUS);
                const double fill = (double)std::min<int64_t>(wgs, CUS) / CUS;
                const double t_stage = t_lo + (t_hi - t_lo) * std::max(0.0, (fill - knee) / (1.0 - knee));
                return std::max(rounds * (double)stages * t_stage + 3.0, stream) + second_pass(sl);
            };
            const double cost1 = cost(slabs, true);
            int64_t s0 = 1, s3 = 1;
            const double cost0 = one_per_cu((O + 255) / 256 * ((I + 255) / 256), 0.44, 0.56, 0.0, s0);       // 256 x 256, 8 waves
            const double cost3 = one_per_cu((O + 255) / 256 * ((I + 127) / 128), 0.30, 0.365, 0.75, s3);     // 256 x 128, 8 waves
            // (with fewer than 32 of its tiles the 256 x 128 plan needs more than eight slabs and measured slower than predicted)
            const int64_t tiles3 = (O + 255) / 256 * ((I + 127) / 128);
            const bool take0 = cost0 < 0.85 * cost1, take3 = tiles3 >= 32 && cost3 < 0.95 * cost1;
            if (take0 && (!take3 || cost0 <= cost3)) {
                p.shape = 0; p.tm = 256; p.tn = 256;
                slabs = (int)s0;
            } else if (take3) {
                p.shape = 3; p.tm = 256; p.tn = 128;
                slabs = (int)s3;
            }
            p.tiles_m = (int)((O + p.tm - 1) / p.tm);
            p.tiles_n = (int)((I + p.tn - 1) / p.tn);
        }
    }
    p.slabs = slabs;
    p.groups_per_slab = slab_groups(groups, p.slabs, 12);                    // whole trips of six LDS stages (2 groups each)
    return p;
}

size_t update_gemm_smfmac_workspace(int64_t T, int64_t O, int64_t I)
{
    if (T <= 0 || O <= 0 || I <= 0) return 0;
    return splitk_workspace_bytes(make_plan(T, O, I).slabs, O, I);
}

size_t update_gemm_smfmac_shifted_workspace(int64_t T, int64_t O, int64_t I)
{
    if (T <= 0 || O <= 0 || I <= 0) return 0;
    return splitk_workspace_bytes(make_plan(T, O, I, true).slabs, O, I);
}

hipError_t launch_update_gemm_smfmac(const void *vals, const uint16_t *meta, const void *h, int64_t ldh, float *dW,
                                     int64_t lddw, int64_t T, int64_t O, int64_t I, float beta, void *workspace,
                                     hipStream_t st)
{
    const Plan p = make_plan(T, O, I);
    const int accumulate = beta != 0.f;
    const OutTarget tg = splitk_target(p.slabs, dW, lddw, workspace, O, I, accumulate);
    float *out = tg.out;
    const int64_t ldo = tg.ldo, slab_stride = tg.slab_stride;
    const int acc_flag = tg.accumulate;
    if (p.tall_rows > 0) {
        dim3 tall_grid((unsigned)(p.tall_tiles_m * p.tiles_n), 1, 1);
        hipLaunchKernelGGL(update_gemm_smfmac_tall_kernel, tall_grid, dim3(512), 0, st, (const uint16_t *)vals, meta, (const uint16_t *)h,
                           ldh, out, ldo, slab_stride, T / 16, p.groups_per_slab, O, I, p.tall_tiles_m, p.tiles_n, acc_flag,
                           (int64_t)0, p.tall_rows);
        hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return e0;
    }
    if (p.tiles_m > 0) {
        dim3 grid((unsigned)(p.tiles_m * p.tiles_n), 1, (unsigned)p.slabs);
#define NM_LAUNCH(WM, WN, AB, BB)                                                                                     \
    hipLaunchKernelGGL((update_gemm_smfmac_kernel<WM, WN, AB, BB>), grid, dim3(WM * WN * 64), 0, st, (const uint16_t *)vals,   \
                       meta, (const uint16_t *)h, ldh, out, ldo, slab_stride, T / 16, p.groups_per_slab, O, I,         \
                       p.tiles_m, p.tiles_n, acc_flag, p.tall_rows, O, ShiftArg{})
        if (p.shape == 0) NM_LAUNCH(2, 4, 4, 2);
        else if (p.shape == 3) NM_LAUNCH(4, 2, 2, 2);
        else NM_LAUNCH(2, 2, 2, 2);
#undef NM_LAUNCH
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.slabs > 1) e = launch_splitk_reduce((const float *)workspace, p.slabs, dW, lddw, O, I, accumulate, 1.0f, st);
    return e;
}

// dW = beta*dW + decompress(vals, meta)^T [x shifted by rows[0] | x shifted by rows[1] | ...]  (I = n * cb columns).
// Same plan as the plain GEMM of that size, on the kernels that take the shift table (no 384-row tiles).
hipError_t launch_update_gemm_smfmac_shifted(const void *vals, const uint16_t *meta, const void *x, int64_t ldx, int64_t cb,
                                             const int64_t *rows, int n, float *dW, int64_t lddw, int64_t T, int64_t O,
                                             float beta, void *workspace, hipStream_t st)
{
    const int64_t I = cb * n;
    if (O == 0 || I == 0) return hipSuccess;
    const Plan p = make_plan(T, O, I, true);
    const ShiftArg sh = make_shift_arg(cb, rows, n);
    const int accumulate = beta != 0.f;
    const OutTarget tg = splitk_target(p.slabs, dW, lddw, workspace, O, I, accumulate);
    float *out = tg.out;
    const int64_t ldo = tg.ldo, slab_stride = tg.slab_stride;
    const int acc_flag = tg.accumulate;
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), 1, (unsigned)p.slabs);
#define NM_LAUNCH(WM, WN, AB, BB)                                                                                     \
    hipLaunchKernelGGL((update_gemm_smfmac_kernel<WM, WN, AB, BB, true>), grid, dim3(WM * WN * 64), 0, st,              \
                       (const uint16_t *)vals, meta, (const uint16_t *)x, ldx, out, ldo, slab_stride, T / 16,            \
                       p.groups_per_slab, O, I, p.tiles_m, p.tiles_n, acc_flag, (int64_t)0, O, sh)
    if (p.shape == 0) NM_LAUNCH(2, 4, 4, 2);
    else if (p.shape == 1) NM_LAUNCH(2, 2, 2, 2);
    else if (p.shape == 3) NM_LAUNCH(4, 2, 2, 2);
    else NM_LAUNCH(1, 4, 2, 2);
#undef NM_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.slabs > 1) e = launch_splitk_reduce((const float *)workspace, p.slabs, dW, lddw, O, I, accumulate, 1.0f, st);
    return e;
}

}  // namespace nm
