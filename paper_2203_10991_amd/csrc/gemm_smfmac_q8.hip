// Update GEMM on CDNA4 sparse MFMA with 8-bit operands:
//     dW[O x I] = beta*dW + alpha * decompress(vals8, meta32)^T h8        (eq. (3); Sec. 5, 8-bit rows)
// vals8: kept neural-gradient values in e5m2 (32-token group format), h8: activations in e4m3.
//
// Instruction: v_smfmac_f32_32x32x64_bf8_fp8.  Lane layouts, as measured on gfx950 (l = lane):
//   A  lane holds the 16 kept values of row (l%32) for the 32 tokens  32*(l/32) .. +31  of the 64-token
//      step, quad by quad: one 16-byte `vals8` fragment; the 32-bit index register (2 bits per kept value)
//      is exactly one `meta32` word of the group format.
//   B  lane holds column (l%32); bytes 0-15 = tokens 16*(l/32) .. +15, bytes 16-31 = tokens 32 + 16*(l/32) .. +15.
//      h8 is token-major, so the tile is staged in LDS as [token][column] and read with ds_read_b64_tr_b8:
//      per 16 lanes, lane j supplies the address of 8 bytes, and lane i receives byte i%8 of the 8 pieces
//      supplied by lanes i/8, i/8+2, ..., i/8+14.  Lane j supplies token j/2, column half j%2 of a 16-column
//      chunk: lane i then holds column i of the chunk for 8 consecutive tokens.
//   D  reg r of lane l = row 8*(r/4) + 4*(l/32) + r%4, column l%32.
//
// The kernel has the structure of the 16-bit one (same bytes per stage: a stage is 64 tokens of 1-byte
// operands instead of 32 tokens of 2-byte ones): every operand byte of a stage reaches the CU once by direct
// global->LDS loads spread over the stage's MFMAs, six stages rotate through LDS, one bare barrier per stage,
// operand registers double-buffered, split-K with a deterministic second pass.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <type_traits>
#include <utility>

#include "nm_internal.h"
#include "smfmac_common.h"
#include "gemm_plan.h"

namespace nm {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

constexpr int KT8 = 64;           // tokens per LDS stage (one 64-token MFMA step, two 32-token groups)
constexpr int NS8 = 6;            // LDS stages

union FragB8 { i32x8 v; u32x2 q[4]; };
union FragA8 { i32x4 v; u32x4 u4; };

// IN_VGPR: the accumulator block lives in ordinary registers (see acc_zero)
template <bool IN_VGPR = false>
__device__ __forceinline__ void smfmac_32x32x64_bf8_fp8(f32x16 &acc, const i32x4 &a, const i32x8 &b, uint32_t idx)
{
    if constexpr (IN_VGPR) asm volatile("v_smfmac_f32_32x32x64_bf8_fp8 %0, %1, %2, %3" : "+v"(acc) : "v"(a), "v"(b), "v"(idx));
    else                   asm volatile("v_smfmac_f32_32x32x64_bf8_fp8 %0, %1, %2, %3" : "+a"(acc) : "v"(a), "v"(b), "v"(idx));
}
template <int OFFSET> __device__ __forceinline__ void lds_refill_tr8(u32x2 &r, uint32_t addr)
{
    asm volatile("ds_read_b64_tr_b8 %0, %1 offset:%2" : "+v"(r) : "v"(addr), "n"(OFFSET) : "memory");
}
template <int OFFSET> __device__ __forceinline__ void lds_refill_b64(u32x2 &r, uint32_t addr)
{
    asm volatile("ds_read_b64 %0, %1 offset:%2" : "+v"(r) : "v"(addr), "n"(OFFSET) : "memory");
}
// alpha * (one accumulator element) to global memory: the element is copied out of its accumulation register, scaled
// and stored inside one statement, so that the compiler never holds whole blocks in ordinary registers
__device__ __forceinline__ void store_acc_scaled(float *p, float v, float alpha)
{
    float t;
    asm volatile("v_accvgpr_read_b32 %0, %2\n\tv_mul_f32 %0, %0, %3\n\tglobal_store_dword %1, %0, off"
                 : "=&v"(t) : "v"(p), "a"(v), "v"(alpha) : "memory");
}
// The (accumulate, alpha) argument pair of the kernels also carries the device-scale form without another kernel
// argument (the 384 x 256 kernel has no register to spare for one): accumulate bit 0 = add to what is there, bit 1 =
// "the scale is in device memory", and then the other 62 bits of the pair are the address of that binary32 value
// (4-byte aligned: low 30 bits in accumulate[31:2], high 32 bits in alpha's bit pattern).  Decoded in the epilogue only.
__device__ __forceinline__ float decode_alpha(int accumulate, float alpha)
{
    if (accumulate & 2) {
        const uint64_t addr = ((uint64_t)__float_as_uint(alpha) << 32) | (uint32_t)(accumulate & ~3);
        return *(const float *)addr;
    }
    return alpha;
}
template <int OFFSET> __device__ __forceinline__ u32x2 lds_read_tr8(uint32_t addr)
{
    u32x2 r;
    asm volatile("ds_read_b64_tr_b8 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFFSET) : "memory");
    return r;
}

// LDS image of one stage (all filled by direct loads, 64 consecutive lanes -> consecutive LDS bytes):
//   [0, 64*TN)     h8 tile, [64 tokens][TN columns], rows unpadded; 16-byte chunk c of row k sits at chunk position
//                  c ^ (2*(k%8)): a transposing read touches, per 32 lanes, two neighbouring chunks of 8 consecutive rows
//   then           vals8 fragments, [2 token groups][TM slots] x 16 bytes
//   then           meta32 words,   [2 token groups][TM rows]  x 4 bytes
//                  (both as one share per wave, padded to a whole 64-lane load)
// SHIFTED: h8 as row-shifted views of one matrix (see ShiftArg); only a lane's source offset and the descriptor change.
template <int WM, int WN, int AB, int BB, bool SHIFTED = false>
__global__ __launch_bounds__(WM * WN * 64) void update_gemm_smfmac_q8_kernel(
    const uint8_t *__restrict__ vals, const uint32_t *__restrict__ meta, const uint8_t *__restrict__ h, int64_t ldh,
    float *__restrict__ out, int64_t ldo, int64_t slab_stride,
    int64_t n_groups, int64_t groups_per_slab, int64_t O, int64_t I, int tiles_m, int tiles_n, int accumulate, float alpha,
    int64_t o_first,                         // the launch computes rows [o_first, O) of dW; tiles_m counts its M-tiles
    ShiftArg sh)                             // (SHIFTED only)
{
    constexpr int TM = WM * AB * 32, TN = WN * BB * 32;
    static_assert(TN == 256, "the h8 swizzle is written for 16 chunks per row");
    constexpr int CPR = TN / 16;                          // 16-byte chunks per h8 row in LDS
    constexpr int ROWS_PER_DMA = 64 / CPR;                // h8 rows one wave-wide 16-byte direct load covers (4)
    constexpr int NW = WM * WN;
    constexpr int WPG = NW / 2;                           // waves that share one of the stage's 2 token groups
    constexpr int B_ROWS = KT8 / NW;                      // h8 rows a wave brings per stage
    constexpr int A_ROWS = TM / WPG;                      // tile rows a wave brings (vals8 and meta32) of its token group
    constexpr int B_DMA = B_ROWS / ROWS_PER_DMA;
    constexpr int A_DMA = A_ROWS >= 64 ? A_ROWS / 64 : 1; //   vals8: 64 rows (16 bytes each) per load
    constexpr int A_LANES = A_ROWS >= 64 ? 64 : A_ROWS;
    constexpr int A_SLOTS = A_ROWS >= 64 ? A_ROWS : 64;
    constexpr int M_DMA = A_DMA;                          //   meta32: one word per lane
    constexpr int M_SLOTS = A_SLOTS;                      //   4-byte slots per share in LDS
    static_assert(NW == 4 || NW == 8, "4 or 8 waves");
    static_assert(B_DMA >= 1 && B_ROWS % 8 == 0 && A_ROWS >= 16, "tile too small for this wave count");
    constexpr int LOADS_PER_STAGE = B_DMA + A_DMA + M_DMA;
    constexpr int A_OFF = KT8 * TN, M_OFF = A_OFF + 2 * WPG * A_SLOTS * 16;
    constexpr int STAGE_BYTES = (M_OFF + 2 * WPG * M_SLOTS * 4 + 1023) / 1024 * 1024;
    static_assert(NS8 * STAGE_BYTES <= 160 * 1024, "LDS");
    __shared__ __attribute__((aligned(1024))) char S[NS8 * STAGE_BYTES];
    auto buf = [&](auto u_c) -> char * { return S + (decltype(u_c)::value % NS8) * STAGE_BYTES; };

    int tm, tn, slab;
    tile_and_slab_of_workgroup(tiles_m, tiles_n, tm, tn, slab);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int64_t m0 = o_first + (int64_t)tm * TM;
    const int64_t n0 = (int64_t)tn * TN;
    const int64_t g_begin = (int64_t)slab * groups_per_slab;
    const int64_t g_end = min(n_groups, g_begin + groups_per_slab);
    out += (int64_t)slab * slab_stride;

    f32x16 acc[AB][BB];
#pragma unroll
    for (int a = 0; a < AB; ++a)
#pragma unroll
        for (int b = 0; b < BB; ++b) acc_zero(acc[a][b]);

    const int n_iters = (int)((g_end - g_begin + 1) / 2);      // stages of 2 token groups; the last may be ragged

    // Raw buffer descriptors, re-based as the kernel advances: a load from past the end of the tensor (the token
    // group a ragged last stage lacks) is dropped by the bounds check.
    auto rsrc = [](const void *base, int64_t bytes) {
        const uint32_t n = bytes <= 0 ? 0u : (bytes > 0xffffffffll ? 0xffffffffu : (uint32_t)bytes);
        return __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)n, 0x00020000);
    };
    const int64_t T = n_groups * 32;

    // per-lane source offsets (bytes, relative to the stage).  Rows >= O and columns >= I are clamped to the last
    // valid ones: their products land in outputs that are never stored.
    const int wgrp = wave / WPG, wsub = wave % WPG;
    uint32_t a_src[A_DMA], m_src[M_DMA];
#pragma unroll
    for (int d = 0; d < A_DMA; ++d) {
        // LDS slot q of a token group holds tile row slot_row(q): inside each wave-row block of AB*32 rows, the 32 rows
        // that feed accumulator block a (rows a, AB+a, 2AB+a, ...) are stored next to each other
        const int q = wsub * A_ROWS + 64 * d + (lane % A_LANES);
        const int row = (q / (AB * 32)) * (AB * 32) + AB * (q % 32) + (q % (AB * 32)) / 32;
        a_src[d] = (uint32_t)(wgrp * O + min(m0 + row, O - 1)) * 16u;
        // index words stay in natural row order
        m_src[d] = (uint32_t)(wgrp * O + min(m0 + wsub * A_ROWS + 64 * d + (lane % A_LANES), O - 1)) * 4u;
    }
    // h8: direct load d of this wave fills rows  wave*B_ROWS + d*ROWS_PER_DMA + lane/CPR  at chunk position
    // lane%CPR, i.e. it must fetch global chunk  (lane%CPR) ^ 2*(row%8).
    constexpr int PHASES = 8 / ROWS_PER_DMA;
    static_assert(B_DMA % PHASES == 0, "a wave's rows cover whole swizzle periods");
    uint32_t b_src[PHASES];
    const int dma_row = lane / CPR, dma_pos = lane % CPR;
#pragma unroll
    for (int ph = 0; ph < PHASES; ++ph) {
        const int row_mod8 = (ph * ROWS_PER_DMA + dma_row) & 7;
        const int64_t col = min(n0 + 16 * (dma_pos ^ (2 * row_mod8)), I - 16);
        if constexpr (SHIFTED) {
            const int j = (int)(col / sh.cb);             // (a 16-byte chunk never straddles two views: cb % 16 == 0)
            b_src[ph] = (uint32_t)((int64_t)(wave * B_ROWS + dma_row + sh.rows[j] + sh.margin) * ldh + (col - (int64_t)j * sh.cb));
        } else
        b_src[ph] = (uint32_t)((int64_t)(wave * B_ROWS + dma_row) * ldh + col);
    }
    const uint32_t b_row_step = (uint32_t)(ROWS_PER_DMA * ldh);

    __amdgpu_buffer_rsrc_t rh, rv, rm;
    auto rebase = [&](int it) {
        const int64_t Gs = g_begin + (int64_t)it * 2, t0 = Gs * 32;
        if constexpr (SHIFTED)       // offsets are relative to row t0 - margin
            rh = rsrc((const char *)h + (t0 - sh.margin) * ldh, (T - t0 - 1 + 2 * (int64_t)sh.margin) * ldh + sh.cb);
        else
        rh = rsrc((const char *)h + t0 * ldh, (T - t0 - 1) * ldh + I);
        rv = rsrc((const char *)vals + Gs * O * 16, (n_groups - Gs) * O * 16);
        rm = rsrc((const char *)meta + Gs * O * 4, (n_groups - Gs) * O * 4);
    };
    const uint32_t h_stage = (uint32_t)(KT8 * ldh), v_stage = (uint32_t)(2 * O * 16), m_stage = (uint32_t)(2 * O * 4);
    auto fetch_one = [&](auto u_c, auto k_c, char *stage) {
        constexpr uint32_t U = decltype(u_c)::value;
        constexpr int K = decltype(k_c)::value;
        if constexpr (K < B_DMA)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rh, (lptr_t)(stage + (wave * B_ROWS + K * ROWS_PER_DMA) * TN), 16,
                                                     (int)(b_src[K % PHASES] + (uint32_t)K * b_row_step + U * h_stage), 0, 0, 0);
        else if constexpr (K < B_DMA + A_DMA)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rv, (lptr_t)(stage + A_OFF + (wave * A_SLOTS + 64 * (K - B_DMA)) * 16), 16,
                                                     (int)(a_src[K - B_DMA] + U * v_stage), 0, 0, 0);
        else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rm, (lptr_t)(stage + M_OFF + (wave * M_SLOTS + 64 * (K - B_DMA - A_DMA)) * 4), 4,
                                                     (int)(m_src[K - B_DMA - A_DMA] + U * m_stage), 0, 0, 0);
    };
    auto fetch = [&](auto u_c, char *stage) {
        static_for<LOADS_PER_STAGE>([&](auto k_c) { fetch_one(u_c, k_c, stage); });
    };
    // first stage (relative to the slab) in which this wave's token group lies past the end of the tensor
    const int first_missing = (int)min((int64_t)0x7fffffff, (n_groups - g_begin - wgrp + 1) / 2);
    auto stage_ready = [&](auto in_flight_c, int it, char *stage) {
        wait_vmcnt<decltype(in_flight_c)::value * LOADS_PER_STAGE>();
        // a direct load whose source lies past the end of the tensor leaves its LDS bytes untouched: the wave
        // clears what it would have brought
        if (it >= first_missing) {
            const uint4 z = make_uint4(0, 0, 0, 0);
            for (int c = lane; c < B_ROWS * CPR; c += 64) *(uint4 *)(stage + wave * B_ROWS * TN + c * 16) = z;
            for (int c = lane; c < A_SLOTS; c += 64) *(uint4 *)(stage + A_OFF + (wave * A_SLOTS + c) * 16) = z;
            for (int c = lane; c < M_SLOTS / 4; c += 64) *(uint4 *)(stage + M_OFF + wave * M_SLOTS * 4 + c * 16) = z;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };

    // lane's LDS read addresses inside a stage.  h8, read j (0..3) of a fragment covers the tokens
    // 32*(j/2) + 16*(lane/32) + 8*(j%2) .. +7; the lane supplies token li/2 of them, half li%2 of its 16-column chunk.
    const int li = lane & 15, grp = (lane >> 4) & 1, kg = lane >> 5;
    const int rd_row = (16 * kg + (li >> 1)) * TN;
    // The read addresses are registers that walk through the stages (advanced by an asm add after the reads of a
    // stage: the compiler would otherwise keep one copy of every address per stage buffer).
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)S;
    uint32_t cur_b[BB];
#pragma unroll
    for (int b = 0; b < BB; ++b)
        cur_b[b] = lds0 + (uint32_t)(rd_row + ((2 * (wn * BB + b) + grp) ^ (2 * (li >> 1))) * 16 + (li & 1) * 8);
    constexpr int A_BLOCK = (A_ROWS >= 64 ? 32 : 64) * 16;
    static_assert(A_ROWS % 32 == 0 && (AB * 32) % A_ROWS == 0 || A_ROWS % (AB * 32) == 0, "shares and wave rows nest");
    const int q0 = wm * (AB * 32), r0 = q0 + AB * (lane & 31);
    uint32_t cur_a = lds0 + (uint32_t)(A_OFF + ((kg * WPG + q0 / A_ROWS) * A_SLOTS + q0 % A_ROWS + (lane & 31)) * 16);   // + a*A_BLOCK
    uint32_t cur_m = lds0 + (uint32_t)(M_OFF + ((kg * WPG + r0 / A_ROWS) * M_SLOTS + r0 % A_ROWS) * 4);                   // AB consecutive words
    static_assert(BB == 2, "advance() moves two column-fragment addresses");
    auto advance = [&](int bytes) {
        asm volatile("v_add_u32 %0, %4, %0\n\tv_add_u32 %1, %4, %1\n\tv_add_u32 %2, %4, %2\n\tv_add_u32 %3, %4, %3"
                     : "+v"(cur_a), "+v"(cur_m), "+v"(cur_b[0]), "+v"(cur_b[1]) : "s"(bytes));
    };

    static_assert(AB == 2 || AB == 4, "AB is 2 or 4");
    FragA8 af[2][AB];
    u32x4 ix4[2]; u32x2 ix2[2];             // index words as read, AB consecutive 32-bit words
    FragB8 bf[2][BB];
    constexpr int NR = AB + 1 + 4 * BB;
    constexpr int NM = AB * BB;
    static_assert(NR <= 15, "lgkmcnt is a 4-bit counter");
    // read number r of the stage the address registers point at
    auto lds_read = [&](auto set_c, auto r_c) {
        constexpr int set = decltype(set_c)::value, r = decltype(r_c)::value;
        if constexpr (r < AB) af[set][r].u4 = lds_read_b128<r * A_BLOCK>(cur_a);
        else if constexpr (r == AB) {
            if constexpr (AB == 4) ix4[set] = lds_read_b128<0>(cur_m);
            else                   ix2[set] = lds_read_b64<0>(cur_m);
        } else {
            constexpr int j = r - AB - 1, b = j / 4, qd = j % 4;
            bf[set][b].q[qd] = lds_read_tr8<(32 * (qd >> 1) + 8 * (qd & 1)) * TN>(cur_b[b]);
        }
    };
    // NEXT_STEP: what moves the address registers from the stage read here to the one after it
    auto consume = [&](auto set_c, auto next_step_c, auto fu_c, char *far) {
        constexpr int set = decltype(set_c)::value;
        constexpr int NL = LOADS_PER_STAGE;
        if constexpr (AB == 4) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(ix4[set]));
        else                   asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(ix2[set]));
        static_for<NM>([&](auto m_c) {
            constexpr int m = decltype(m_c)::value, b = m / AB, a = m % AB;
            uint32_t idx;
            if constexpr (AB == 4) idx = ix4[set][a];
            else                   idx = ix2[set][a];
            smfmac_32x32x64_bf8_fp8(acc[a][b], af[set][a].v, bf[set][b].v, idx);
            static_for<NR>([&](auto r_c) {
                constexpr int r = decltype(r_c)::value;
                if constexpr (r >= m * NR / NM && r < (m + 1) * NR / NM) lds_read(std::integral_constant<int, 1 - set>{}, r_c);
            });
            static_for<NL>([&](auto k_c) {
                constexpr int k = decltype(k_c)::value;
                if constexpr (k >= m * NL / NM && k < (m + 1) * NL / NM) fetch_one(fu_c, k_c, far);
            });
        });
        advance(decltype(next_step_c)::value);
    };

    // Six LDS stages rotating, straight-line loop body of six stages per trip; stages past the end of the tensor
    // hold zeros (dropped loads, cleared shares), so the stage count is padded to a multiple of six.
    const int n_trips = (n_iters + NS8 - 1) / NS8;
    if (n_trips > 0) {
        rebase(0);
        static_for<NS8 - 1>([&](auto u_c) { fetch(u_c, buf(u_c)); });
        stage_ready(std::integral_constant<int, NS8 - 2>{}, 0, S);
        static_for<NR>([&](auto r_c) { lds_read(std::integral_constant<int, 0>{}, r_c); });
        advance(STAGE_BYTES);
    }
    for (int tr = 0; tr < n_trips; ++tr) {
        const int it = NS8 * tr;
        rebase(it);
        static_for<NS8>([&](auto u_c) {
            constexpr int u = decltype(u_c)::value;
            stage_ready(std::integral_constant<int, NS8 - 3>{}, it + u + 1, buf(std::integral_constant<int, u + 1>{}));
            // the reads issued during stage u are those of stage u+1; the ones after them belong to stage u+2
            consume(std::integral_constant<int, u % 2>{},
                    std::integral_constant<int, ((u + 2) % NS8 == 0) ? -(NS8 - 1) * STAGE_BYTES : STAGE_BYTES>{},
                    std::integral_constant<int, u + NS8 - 1>{}, buf(std::integral_constant<int, u + NS8 - 1>{}));
        });
    }

    // ---- epilogue: idle for longer than an 8-pass instruction before the first read of an accumulation register,
    // and tie every such read behind that wait (the compiler cannot see MFMAs inside asm statements)
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
    for (int a = 0; a < AB; ++a)
#pragma unroll
        for (int b = 0; b < BB; ++b) acc_settled(acc[a][b]);
    __builtin_amdgcn_sched_barrier(0);
    const float alpha_v = decode_alpha(accumulate, alpha);
    const int64_t o0 = m0 + wm * (AB * 32);
#pragma unroll
    for (int a = 0; a < AB; ++a)
#pragma unroll
        for (int b = 0; b < BB; ++b) {
            const int64_t col = n0 + wn * (BB * 32) + b * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = o0 + AB * (8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) + a;   // block a holds rows a, AB+a, ...
                if (row < O && col < I) {
                    float *p = out + row * ldo + col;
                    if (accumulate & 1) *p = *p + acc[a][b][r] * alpha_v;
                    else store_acc_scaled(p, acc[a][b][r], alpha_v);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
}

// ------------------------------------------------------------------------------------
// 384 x 256 tile for large problems (the 8-bit kernels are bound by the path from the L2s to the CUs; a tile that is
// 1.5 times taller needs 21 % fewer operand bytes per product).  Same construction as the 16-bit 384 x 256 kernel:
// 8 waves as 2 x 4, wave tile 192 x 64 = 6 x 2 accumulator blocks, four of the six row blocks in accumulation
// registers and two in ordinary ones, single operand registers refilled in place right after the last MFMA that
// reads them, five stages of 31 KB, rows of a wave's block interleaved by six (block a holds rows 6m + a) so that a
// lane's six index words are adjacent.  Differences: a stage is 64 one-byte tokens; the index words are 32-bit
// (three ds_read_b64 per lane and stage); h8 goes through ds_read_b64_tr_b8 with the swizzle c ^ 2(k%8), under
// which the wave's second column block (8 chunks further) sits at the first one's address with bit 7 flipped.
// No split-K: this kernel only serves problems with at least a GPU-wide round of its tiles.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void update_gemm_smfmac_q8_tall_kernel(
    const uint8_t *__restrict__ vals, const uint32_t *__restrict__ meta, const uint8_t *__restrict__ h, int64_t ldh,
    float *__restrict__ out, int64_t ldo, int64_t n_groups, int64_t O, int64_t I, int tiles_m, int tiles_n,
    int accumulate, float alpha, int64_t o_end)          // rows [0, o_end) of dW
{
    constexpr int WN = 4, AB = 6, BB = 2, TM = 384, TN = 256, TNS = 5;
    constexpr int A_OFF = KT8 * TN, M_OFF = A_OFF + 2 * TM * 16, STAGE = (M_OFF + 2 * TM * 4 + 1023) / 1024 * 1024;
    constexpr int LPS = 6;                                   // direct loads per wave and stage: 2 h8, 2 vals8, 2 meta32
    static_assert(TNS * STAGE <= 160 * 1024 && STAGE % 256 == 0, "LDS");
    __shared__ __attribute__((aligned(1024))) char S[TNS * STAGE];

    int tm, tn;
    tile_of_workgroup((int)blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int64_t m0 = (int64_t)tm * TM, n0 = (int64_t)tn * TN;

    f32x16 acc[AB][BB];
    static_for<AB>([&](auto a_c) {
        constexpr int a = decltype(a_c)::value;
        static_for<BB>([&](auto b_c) { acc_zero<(a >= 4)>(acc[a][decltype(b_c)::value]); });
    });

    const int n_iters = (int)((n_groups + 1) / 2);           // stages of 2 token groups; the last may be ragged
    const int n_trips = (n_iters + TNS - 1) / TNS;

    auto slot_row = [](int q) {                               // tile row held by slot q of a token group
        const int blk = q / 192, r = q % 192, a = r / 32, m = r % 32;
        return blk * 192 + 6 * m + a;
    };
    // ---- direct loads.  Wave w brings, of token group w/4 of the stage: 8 rows of h8 (2 loads), vals8 slots and
    // meta32 rows [96*(w%4), +96) as one 64-lane and one 32-lane load each.  Per-lane byte offsets inside a stage;
    // the stage is reached through the scalar offset, which the bounds check does not cover: a load for a token
    // group past the end of the tensor is switched off through the descriptor's size instead.
    const int wgrp = wave / 4, ws = wave % 4;
    uint32_t b_src[2], a_src[2], m_src[2];
    {
        constexpr int CPR = TN / 16;                         // 16 chunks of 16 bytes per h8 row
        const int dma_row = lane / CPR, dma_pos = lane % CPR;
#pragma unroll
        for (int ph = 0; ph < 2; ++ph) {                     // load ph covers rows 8*wave + 4*ph + dma_row
            const int row_mod8 = (4 * ph + dma_row) & 7;
            const int64_t col = min(n0 + 16 * (dma_pos ^ (2 * row_mod8)), I - 16);
            b_src[ph] = (uint32_t)((int64_t)(wave * 8 + 4 * ph + dma_row) * ldh + col);
        }
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            const int q = 96 * ws + 64 * d + (d ? (lane & 31) : lane);
            a_src[d] = (uint32_t)(wgrp * O + min(m0 + slot_row(q), O - 1)) * 16u;
            m_src[d] = (uint32_t)(wgrp * O + min(m0 + q, O - 1)) * 4u;
        }
    }
    const bool lane_lt32 = lane < 32;
    const uint32_t h_stage = (uint32_t)(KT8 * ldh), v_stage = (uint32_t)(2 * O * 16), m_stage = (uint32_t)(2 * O * 4);
    const int first_missing = (int)min((int64_t)0x7fffffff, (n_groups - wgrp + 1) / 2);
    const char *hp = nullptr, *vp = nullptr, *mp = nullptr;   // the tensors at the first stage of the current trip
    int trip_first = 0;
    auto rebase = [&](int it) {
        const int64_t Gs = (int64_t)it * 2;
        hp = (const char *)h + Gs * 32 * ldh;
        vp = (const char *)vals + Gs * O * 16;
        mp = (const char *)meta + Gs * O * 4;
        trip_first = it;
    };
    auto fetch_one = [&](auto u_c, auto k_c, auto buf_c) {
        constexpr uint32_t U = decltype(u_c)::value;
        constexpr int K = decltype(k_c)::value, BUF = decltype(buf_c)::value % TNS;
        const int size = trip_first + (int)U < first_missing ? 0x7fffffff : 0;        // 0: nothing is loaded
        char *stage = S + BUF * STAGE;
        if constexpr (K < 2)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(__builtin_amdgcn_make_buffer_rsrc((void *)hp, 0, size, 0x00020000),
                                                     (lptr_t)(stage + (wave * 8 + 4 * K) * TN), 16, (int)b_src[K],
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
        } else if constexpr (K == 4)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(__builtin_amdgcn_make_buffer_rsrc((void *)mp, 0, size, 0x00020000),
                                                     (lptr_t)(stage + M_OFF + (wgrp * TM + 96 * ws) * 4), 4, (int)m_src[0],
                                                     (int)(U * m_stage), 0, 0);
        else {
            if (lane_lt32)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(__builtin_amdgcn_make_buffer_rsrc((void *)mp, 0, size, 0x00020000),
                                                         (lptr_t)(stage + M_OFF + (wgrp * TM + 96 * ws + 64) * 4), 4,
                                                         (int)m_src[1], (int)(U * m_stage), 0, 0);
        }
    };
    // "stage `it` has landed"; a wave whose token group lies past the end of the tensor clears the kept values and
    // the h8 rows it would have brought (its loads were switched off; index words may hold anything)
    auto stage_ready = [&](auto in_flight_c, int it, auto buf_c) {
        constexpr int BUF = decltype(buf_c)::value % TNS;
        wait_vmcnt<decltype(in_flight_c)::value * LPS>();
        if (it >= first_missing) {
            char *stage = S + BUF * STAGE;
            uint32_t zero, ln;
            asm volatile("v_mov_b32 %0, 0\n\tv_mbcnt_lo_u32_b32 %1, -1, 0\n\tv_mbcnt_hi_u32_b32 %1, -1, %1" : "=v"(zero), "=v"(ln));
            const uint4 z = make_uint4(zero, zero, zero, zero);
            *(uint4 *)(stage + A_OFF + (wgrp * TM + 96 * ws + ln) * 16) = z;
            if (ln < 32) *(uint4 *)(stage + A_OFF + (wgrp * TM + 96 * ws + 64 + ln) * 16) = z;
            *(uint4 *)(stage + wave * 8 * TN + ln * 16) = z;
            *(uint4 *)(stage + wave * 8 * TN + 1024 + ln * 16) = z;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- LDS read addresses of the stage being read; they advance by one stage per slot
    const int li = lane & 15, grp = (lane >> 4) & 1, kg = lane >> 5, m = lane & 31;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)S;
    uint32_t cur_a = lds0 + (uint32_t)(A_OFF + (kg * TM + wm * 192 + m) * 16);                 // + 32*a*16
    uint32_t cur_m = lds0 + (uint32_t)(M_OFF + (kg * TM + wm * 192 + 6 * m) * 4);              // 6 consecutive words (three reads)
    // column block b of wave wn is block b*4 + wn of the tile, chunks 8b + 2wn + {0,1}: block 1 = block 0 with bit 7
    // of the address flipped (every stage starts on a multiple of 256 bytes)
    uint32_t cur_b = lds0 + (uint32_t)((16 * kg + (li >> 1)) * TN + ((2 * wn + grp) ^ (2 * (li >> 1))) * 16 + (li & 1) * 8);
    auto advance = [&](int bytes) {
        asm volatile("v_add_u32 %0, %3, %0\n\tv_add_u32 %1, %3, %1\n\tv_add_u32 %2, %3, %2" : "+v"(cur_a), "+v"(cur_m), "+v"(cur_b) : "s"(bytes));
    };

    FragA8 af[AB];
    FragB8 bf[BB];
    u32x2 ix[3] = {u32x2{0, 0}, u32x2{0, 0}, u32x2{0, 0}};   // index words of blocks (0,1), (2,3), (4,5)
#pragma unroll
    for (int a = 0; a < AB; ++a) af[a].u4 = u32x4{0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < BB; ++b)
#pragma unroll
        for (int j = 0; j < 4; ++j) bf[b].q[j] = u32x2{0, 0};
    auto read_a = [&](auto a_c) { constexpr int a = decltype(a_c)::value; lds_refill_b128<32 * a * 16>(af[a].u4, cur_a); };
    auto read_ix = [&](auto j_c) { constexpr int j = decltype(j_c)::value; lds_refill_b64<8 * j>(ix[j], cur_m); };
    auto read_b = [&](auto b_c) {
        constexpr int b = decltype(b_c)::value;
        uint32_t addr = cur_b;
        if constexpr (b == 1) asm volatile("v_xor_b32 %0, 0x80, %1" : "=v"(addr) : "v"(cur_b));
        lds_refill_tr8<0 * TN>(bf[b].q[0], addr);
        lds_refill_tr8<8 * TN>(bf[b].q[1], addr);
        lds_refill_tr8<32 * TN>(bf[b].q[2], addr);
        lds_refill_tr8<40 * TN>(bf[b].q[3], addr);
    };
    // LDS reads of one stage, in issue order (the waits below count on it):
    //   B0 (4 reads) | A0 | A1, ix0 | A2 | A3, ix1 | A4 | A5, ix2, B1 (4)
    auto mfma = [&](auto a_c, auto b_c) {
        constexpr int a = decltype(a_c)::value, b = decltype(b_c)::value;
        smfmac_32x32x64_bf8_fp8<(a >= 4)>(acc[a][b], af[a].v, bf[b].v, ix[a / 2][a & 1]);
    };
    auto lgkm_wait = [&](auto n_c) { asm volatile("s_waitcnt lgkmcnt(%0)" : : "n"(decltype(n_c)::value)); };
    using I0 = std::integral_constant<int, 0>; using I1 = std::integral_constant<int, 1>; using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>; using I4 = std::integral_constant<int, 4>; using I5 = std::integral_constant<int, 5>;
    auto consume = [&](auto fu_c, auto fbuf_c) {
        lgkm_wait(std::integral_constant<int, 10>{}); mfma(I0{}, I0{});
        fetch_one(fu_c, I0{}, fbuf_c);
        mfma(I1{}, I0{});
        lgkm_wait(std::integral_constant<int, 7>{});  mfma(I2{}, I0{});
        fetch_one(fu_c, I1{}, fbuf_c);
        mfma(I3{}, I0{});
        lgkm_wait(std::integral_constant<int, 4>{});  mfma(I4{}, I0{});           // (ix2 is the last read before B1)
        fetch_one(fu_c, I2{}, fbuf_c);
        mfma(I5{}, I0{});
        read_b(I0{});
        asm volatile("s_waitcnt lgkmcnt(4)");
        mfma(I0{}, I1{}); read_a(I0{});
        fetch_one(fu_c, I3{}, fbuf_c);
        mfma(I1{}, I1{}); read_a(I1{}); read_ix(I0{});
        mfma(I2{}, I1{}); read_a(I2{});
        fetch_one(fu_c, I4{}, fbuf_c);
        mfma(I3{}, I1{}); read_a(I3{}); read_ix(I1{});
        mfma(I4{}, I1{}); read_a(I4{});
        fetch_one(fu_c, I5{}, fbuf_c);
        mfma(I5{}, I1{}); read_a(I5{}); read_ix(I2{}); read_b(I1{});
    };
    auto read_all = [&]() {
        read_b(I0{}); read_a(I0{}); read_a(I1{}); read_ix(I0{}); read_a(I2{}); read_a(I3{}); read_ix(I1{}); read_a(I4{});
        read_a(I5{}); read_ix(I2{}); read_b(I1{});
    };

    // Five LDS stages.  Slot j: stage j's operands are in (or on their way into) registers, read during slot j-1;
    // stage j+1 has landed (the barrier that opens the slot) and is read during the slot; the loads of stages j+2 and
    // j+3 are in flight, those of stage j+4 are issued into the buffer stage j-1 occupied.  Stages past the end of
    // the tensor hold zeros, so the stage count is padded to a multiple of five.
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
            advance(u == TNS - 2 ? -(TNS - 1) * STAGE : STAGE);
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
    const float alpha_v = decode_alpha(accumulate, alpha);
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
                    if (accumulate & 1) *p = *p + acc[a][b][r] * alpha_v;
                    else if constexpr (a >= 4) *p = acc[a][b][r] * alpha_v;
                    else store_acc_scaled(p, acc[a][b][r], alpha_v);
                }
            }
            __builtin_amdgcn_sched_barrier(0);       // one block at a time
        }
    });
}

// ------------------------------------------------------------------------------------
// host side: tile shape and split-K plan (pure function of the problem size)
// ------------------------------------------------------------------------------------
// tall_rows: rows [0, tall_rows) of dW are computed by the 384 x 256 kernel (tall_tiles_m tile rows), the rest by the
// kernel of `shape`
struct PlanQ8 { int shape; int tm; int tiles_m, tiles_n; int slabs; int64_t groups_per_slab; int64_t tall_rows; int tall_tiles_m; };

static PlanQ8 make_plan_q8(int64_t T, int64_t O, int64_t I, bool shifted = false)
{
    PlanQ8 p;
    const int64_t groups = T / 32;
    const int CUS = 256;
    // shape 0: 256x256 (8 waves), shape 1: 128x256 (8 waves of 64x64; measured 10-17 % faster than 4 waves of 128x64),
    // shape 2: 64x256 (4 waves)
    p.tall_rows = 0; p.tall_tiles_m = 0;
    if (O <= 64) { p.shape = 2; p.tm = 64; }
    else if ((O + 255) / 256 * ((I + 255) / 256) >= CUS) {
        p.shape = 0; p.tm = 256;
        // rows split between the 384 x 256 and the 256 x 256 kernel as in the 16-bit path; a round of tall tiles takes
        // 1.36 times as long here (measured: 412 us against 302 us per round)
        const RowSplit rs = split_rows_tall(O, I, 1.36, !shifted);
        p.tall_tiles_m = rs.tall_tiles_m;
        p.tall_rows = rs.tall_rows;
    }
    // Mid-sized problems stay on the 256 x 256 kernel once 128 x 256 tiles would need a second round (more than 256 of
    // them): measured on operands that are in no cache, 144 and 192 tiles of 256 x 256 in one round are 14-32 % faster
    // than twice as many 128 x 256 tiles, which need twice the bytes of `h` per product.  Up to 256 tiles of 128 x 256
    // (cut into slabs until every CU has one) the smaller tile on 8 waves is the faster one (5-20 %).
    // With a long reduction (16384 tokens or more) the larger tile also wins from 48 tiles on (the transformer-MLP
    // shape, 64 tiles in four slabs: 78 against 89 us cold): the second pass over its partial sums weighs less.
    else if (!shifted && ((O + 127) / 128 * ((I + 255) / 256) > CUS ||
                          (T >= 16384 && (O + 255) / 256 * ((I + 255) / 256) >= 48))) { p.shape = 0; p.tm = 256; }
    else { p.shape = 1; p.tm = 128; }
    p.tiles_m = (int)((O - p.tall_rows + p.tm - 1) / p.tm);
    p.tiles_n = (int)((I + 255) / 256);
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    // few tiles: the reduction axis is cut into slabs until every CU has one workgroup (these kernels fit one per CU;
    // more slabs than that only lengthen the second pass over the partial sums)
    int slabs = 1;
    if (p.tall_rows == 0 && tiles < CUS && groups >= 24) {
        slabs = (int)(CUS / tiles);
        const int64_t max_slabs = groups / 12;                         // at least 384 tokens per slab
        if (slabs > max_slabs) slabs = (int)max_slabs;
        if (slabs < 1) slabs = 1;
    }
    p.slabs = slabs;
    p.groups_per_slab = slab_groups(groups, p.slabs, 12);              // whole trips of six LDS stages (2 groups each)
    return p;
}

// alpha = rec_a[1] * rec_b[1], left in rec_b[3] (the consumer's scratch slot of a scale record) for the kernels
__global__ void q8_alpha_product_kernel(const float *rec_a, float *rec_b)
{
    if (threadIdx.x == 0) rec_b[3] = rec_a[1] * rec_b[1];
}

// the (accumulate, alpha) pair the kernels take: host scale, or the address of the device scale (see decode_alpha)
struct AlphaPair { int acc; float alpha; };
static AlphaPair encode_alpha(int accumulate, const AlphaArg &al, hipStream_t st)
{
    if (!al.inv_a) return AlphaPair{accumulate, al.value};
    float *slot = const_cast<float *>(al.inv_b) + 3;
    hipLaunchKernelGGL(q8_alpha_product_kernel, dim3(1), dim3(64), 0, st, al.inv_a, const_cast<float *>(al.inv_b));
    const uint64_t addr = (uint64_t)(uintptr_t)slot;
    AlphaPair p;
    p.acc = (int)((uint32_t)addr | 2u | (uint32_t)(accumulate & 1));
    const uint32_t hi = (uint32_t)(addr >> 32);
    __builtin_memcpy(&p.alpha, &hi, 4);
    return p;
}

size_t update_gemm_q8_workspace(int64_t T, int64_t O, int64_t I)
{
    if (T <= 0 || O <= 0 || I <= 0) return 0;
    return splitk_workspace_bytes(make_plan_q8(T, O, I).slabs, O, I);
}

hipError_t launch_update_gemm_q8(const uint8_t *vals8, const uint32_t *meta32, const uint8_t *h8, int64_t ldh, float *dW,
                                 int64_t lddw, int64_t T, int64_t O, int64_t I, AlphaArg alpha, float beta, void *workspace,
                                 hipStream_t st)
{
    if (O == 0 || I == 0) return hipSuccess;
    const PlanQ8 p = make_plan_q8(T, O, I);
    const int accumulate = beta != 0.f;
    const OutTarget tg = splitk_target(p.slabs, dW, lddw, workspace, O, I, accumulate);
    float *out = tg.out;
    const int64_t ldo = tg.ldo, slab_stride = tg.slab_stride;
    // partial sums are scaled once, in the second pass; otherwise the kernels scale, by a host or a device value
    const AlphaPair ap = p.slabs > 1 ? AlphaPair{tg.accumulate, 1.0f} : encode_alpha(tg.accumulate, alpha, st);
    const int acc_flag = ap.acc;
    const float k_alpha = ap.alpha;
    if (p.tall_rows > 0) {
        hipLaunchKernelGGL(update_gemm_smfmac_q8_tall_kernel, dim3((unsigned)(p.tall_tiles_m * p.tiles_n)), dim3(512), 0, st,
                           vals8, meta32, h8, ldh, out, ldo, T / 32, O, I, p.tall_tiles_m, p.tiles_n, acc_flag, k_alpha, p.tall_rows);
        hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return e0;
        if (p.tiles_m == 0) return hipSuccess;
    }
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), 1, (unsigned)p.slabs);
#define NM_LAUNCH(WM, WN, AB, BB)                                                                                     \
    hipLaunchKernelGGL((update_gemm_smfmac_q8_kernel<WM, WN, AB, BB>), grid, dim3(WM * WN * 64), 0, st, vals8, meta32, h8,    \
                       ldh, out, ldo, slab_stride, T / 32, p.groups_per_slab, O, I, p.tiles_m, p.tiles_n, acc_flag, k_alpha,  \
                       p.tall_rows, ShiftArg{})
    if (p.shape == 0) NM_LAUNCH(2, 4, 4, 2);
    else if (p.shape == 1) NM_LAUNCH(2, 4, 2, 2);
    else NM_LAUNCH(1, 4, 2, 2);
#undef NM_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.slabs > 1) e = launch_splitk_reduce((const float *)workspace, p.slabs, dW, lddw, O, I, accumulate, alpha, st);
    return e;
}

size_t update_gemm_q8_shifted_workspace(int64_t T, int64_t O, int64_t I)
{
    if (T <= 0 || O <= 0 || I <= 0) return 0;
    return splitk_workspace_bytes(make_plan_q8(T, O, I, true).slabs, O, I);
}

// dW = beta*dW + alpha * decompress(vals8, meta32)^T [x8 shifted by rows[0] | x8 shifted by rows[1] | ...]
hipError_t launch_update_gemm_q8_shifted(const uint8_t *vals8, const uint32_t *meta32, const uint8_t *x8, int64_t ldx, int64_t cb,
                                         const int64_t *rows, int n, float *dW, int64_t lddw, int64_t T, int64_t O,
                                         AlphaArg alpha, float beta, void *workspace, hipStream_t st)
{
    const int64_t I = cb * n;
    if (O == 0 || I == 0) return hipSuccess;
    const PlanQ8 p = make_plan_q8(T, O, I, true);
    const ShiftArg sh = make_shift_arg(cb, rows, n);
    const int accumulate = beta != 0.f;
    const OutTarget tg = splitk_target(p.slabs, dW, lddw, workspace, O, I, accumulate);
    float *out = tg.out;
    const int64_t ldo = tg.ldo, slab_stride = tg.slab_stride;
    // partial sums are scaled once, in the second pass; otherwise the kernels scale, by a host or a device value
    const AlphaPair ap = p.slabs > 1 ? AlphaPair{tg.accumulate, 1.0f} : encode_alpha(tg.accumulate, alpha, st);
    const int acc_flag = ap.acc;
    const float k_alpha = ap.alpha;
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), 1, (unsigned)p.slabs);
#define NM_LAUNCH(WM, WN, AB, BB)                                                                                     \
    hipLaunchKernelGGL((update_gemm_smfmac_q8_kernel<WM, WN, AB, BB, true>), grid, dim3(WM * WN * 64), 0, st, vals8, meta32, x8, \
                       ldx, out, ldo, slab_stride, T / 32, p.groups_per_slab, O, I, p.tiles_m, p.tiles_n, acc_flag, k_alpha,   \
                       (int64_t)0, sh)
    if (p.shape == 0) NM_LAUNCH(2, 4, 4, 2);
    else if (p.shape == 1) NM_LAUNCH(2, 4, 2, 2);
    else NM_LAUNCH(1, 4, 2, 2);
#undef NM_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.slabs > 1) e = launch_splitk_reduce((const float *)workspace, p.slabs, dW, lddw, O, I, accumulate, alpha, st);
    return e;
}

}  // namespace nm
