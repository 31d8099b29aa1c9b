// Update GEMM on CDNA4 sparse MFMA:  dW[O x I] (+)= decompress(vals, meta)^T h   (eq. (3)).
//
// Instruction: v_smfmac_f32_32x32x32_bf16.  "A" is the 4:2-sparse operand (rows = columns o of
// g, i.e. rows of dW), "B" the dense one (h), both reduced over tokens.  Lane layouts, as
// measured on gfx950 (l = lane):
//   A  lane holds 8 kept values of row (l%32) for the 16 tokens  16*(l/32) .. +15  of the
//      32-token step, quad by quad; the 16-bit index word (2 bits per kept value, ABID selects
//      the half of the index register) is exactly one `meta` word of the group format, and the
//      8 values are one 16-byte `vals` fragment: both are loaded straight from global memory.
//   B  lane holds column (l%32); slots 0-7 = tokens 8*(l/32) .. +7, slots 8-15 = tokens
//      16 + 8*(l/32) .. +7.  h is token-major in memory, so the tile is staged in LDS as
//      [token][column] and read with ds_read_b64_tr_b16 (a 4-token x 16-column transpose per
//      16 lanes).
//   D  reg r of lane l = row 8*(r/4) + 4*(l/32) + r%4, column l%32.
//
// Workgroup = 4 waves (WM x WN), each wave owns AB x BB blocks of 32x32; 64 tokens per LDS
// stage, three stages in flight, one barrier per stage.  Split-K over blockIdx.z writes binary32
// partials that a second kernel sums in a fixed order (deterministic; no atomics).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "nm_internal.h"

namespace nm {

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int KT = 64;            // tokens per LDS stage (two 32-token MFMA steps)

union Frag16 { bf16x16 v; s16x4 q[4]; };
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
union Frag8 { bf16x8 v; u32x4 u4; };

typedef const __attribute__((address_space(1))) void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

// The 16 accumulator blocks of a wave (256 registers) must own the accumulation-register half
// (AGPRs) of the register file for the whole kernel, with everything else in VGPRs.  Left to
// itself the compiler keeps accumulators in VGPRs and shuffles blocks to and from AGPRs around
// every MFMA, so each definition of an accumulator is an asm statement with an AGPR operand:
//   acc_zero   D = 0*0 + 0 with a dense MFMA (inline-constant C), the only way to write 16 AGPRs at once
//   smfmac     D += A(4:2 sparse, index word in the low half of idx) * B
__device__ __forceinline__ void acc_zero(f32x16 &acc)
{
    const bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %1, 0" : "=a"(acc) : "v"(z));
}
//   LGKM > 0: first wait until at most LGKM-1 LDS reads are outstanding (the fragment's own reads are done)
template <int LGKM>
__device__ __forceinline__ void smfmac_32x32x32(f32x16 &acc, const bf16x8 &a, const bf16x16 &b, uint32_t idx)
{
    if (LGKM == 0)
        asm volatile("v_smfmac_f32_32x32x32_bf16 %0, %1, %2, %3" : "+a"(acc) : "v"(a), "v"(b), "v"(idx));
    else if (LGKM == 1)
        asm volatile("s_waitcnt lgkmcnt(0)\n\tv_smfmac_f32_32x32x32_bf16 %0, %1, %2, %3" : "+a"(acc) : "v"(a), "v"(b), "v"(idx));
    else
        asm volatile("s_waitcnt lgkmcnt(4)\n\tv_smfmac_f32_32x32x32_bf16 %0, %1, %2, %3" : "+a"(acc) : "v"(a), "v"(b), "v"(idx));
}

// Transposing LDS read (4 tokens x 16 columns per 16 lanes -> 4 consecutive tokens of one column per
// lane).  Issued as asm so that the compiler does not order it against the direct global->LDS loads
// still in flight for later stages: that ordering is explicit (wait_vmcnt + barrier per stage).
template <int OFFSET>
__device__ __forceinline__ s16x4 lds_read_tr16(uint32_t addr)
{
    s16x4 r;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFFSET) : "memory");
    return r;
}

// s_waitcnt vmcnt(N) only (expcnt / lgkmcnt left at their maxima): at most N vector-memory loads still in flight
template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// LDS image of a stage of h: [KT tokens][TN columns] bf16, rows unpadded (TN*2 bytes).  It is filled by
// direct global->LDS loads (each wave instruction lands 64 consecutive 16-byte chunks), so bank
// conflicts of the transposing reads are avoided by a swizzle instead of padding: chunk c of row k
// lives at chunk position c ^ (4 * (k % 4)).  A transposing read touches, per 16 lanes, the same
// 32-byte column window of 4 consecutive rows; the swizzle spreads those over distinct banks.
template <int WM, int WN, int AB, int BB>
__global__ __launch_bounds__(256) void update_gemm_smfmac_kernel(
    const uint16_t *__restrict__ vals, const uint16_t *__restrict__ meta, const uint16_t *__restrict__ h, int64_t ldh,
    float *__restrict__ out, int64_t ldo, int64_t slab_stride,       // out + z*slab_stride
    int64_t n_groups, int64_t groups_per_slab, int64_t O, int64_t I, int tiles_m, int tiles_n, int accumulate)
{
    constexpr int TM = WM * AB * 32, TN = WN * BB * 32;
    constexpr int CPR = TN / 8;                           // 16-byte chunks per LDS row
    constexpr int ROWS_PER_DMA = 64 / CPR;                // rows one wave-wide direct load covers
    constexpr int DMA_PER_WAVE = KT / (4 * ROWS_PER_DMA); // direct loads per wave per stage
    constexpr int STAGE_BYTES = KT * TN * 2;
    static_assert(CPR >= 16 && CPR <= 64, "tile width");
    // two separate arrays (not one array of two stages): the compiler then knows that a direct load
    // into one buffer cannot alias the LDS reads of the other and leaves those loads in flight
    __shared__ __attribute__((aligned(1024))) char Bs0[STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char Bs1[STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char Bs2[STAGE_BYTES];

    // ---- tile assignment.  Workgroups go round-robin over the 8 XCDs (each has its own L2):
    // give every XCD a contiguous run of tiles, walked N-fastest inside bands of 8 M-tiles.
    const int n_tiles = tiles_m * tiles_n;
    int bid = blockIdx.x;
    {
        const int per_xcd = (n_tiles + 7) / 8;
        const int remapped = (bid % 8) * per_xcd + bid / 8;
        if (n_tiles % 8 == 0) bid = remapped;
    }
    constexpr int BAND = 8;
    const int band = bid / (BAND * tiles_n);
    const int band_rows = min(BAND, tiles_m - band * BAND);
    const int in_band = bid - band * BAND * tiles_n;
    const int tm = band * BAND + in_band % band_rows;
    const int tn = in_band / band_rows;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);       // wave-uniform: keeps LDS bases scalar
    const int wm = wave / WN, wn = wave % WN;
    const int64_t o0 = (int64_t)tm * TM + wm * (AB * 32);
    const int64_t n0 = (int64_t)tn * TN;                 // tile's first column of h / dW
    const int64_t g_begin = (int64_t)blockIdx.z * groups_per_slab;
    const int64_t g_end = min(n_groups, g_begin + groups_per_slab);
    out += (int64_t)blockIdx.z * slab_stride;

    f32x16 acc[AB][BB];
#pragma unroll
    for (int a = 0; a < AB; ++a)
#pragma unroll
        for (int b = 0; b < BB; ++b) acc_zero(acc[a][b]);

    const int n_iters = (int)((g_end - g_begin + 3) / 4);      // stages of 4 token groups; the last may be ragged

    // All global reads go through raw buffer descriptors that are re-based to the current stage:
    // a 32-bit per-lane offset is all a load needs, and whatever lies past the end of the tensor
    // (the token groups a ragged last stage lacks) reads as zero, so there is no tail code path.
    // Split-K slabs are whole stages except the last, so a ragged stage only occurs at the tensor's end.
    auto rsrc = [](const void *base, int64_t bytes) {
        const uint32_t n = bytes <= 0 ? 0u : (bytes > 0xffffffffll ? 0xffffffffu : (uint32_t)bytes);
        return __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)n, 0x00020000);
    };
    const int64_t T = n_groups * 16;

    // ---- sparse operand: straight from global memory into MFMA registers ---------------------
    // Rows >= O are clamped to the last valid row (their outputs are never stored).
    const int kg = lane >> 5;                                  // which 16-token group of a 32-token step
    uint32_t a_voff[2][AB];                                    // ((2*ks + kg)*O + row)*16: byte offset of the fragment in the stage
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int a = 0; a < AB; ++a)
            a_voff[ks][a] = (uint32_t)((2 * ks + kg) * O + min(o0 + a * 32 + (lane & 31), O - 1)) * 16u;

    auto load_a = [&](int it, Frag8 (&af)[2][AB], uint32_t (&ix)[2][AB]) {
        const int64_t Gs = g_begin + (int64_t)it * 4;
        const __amdgpu_buffer_rsrc_t rv = rsrc((const char *)vals + Gs * O * 16, (n_groups - Gs) * O * 16);
        const __amdgpu_buffer_rsrc_t rm = rsrc((const char *)meta + Gs * O * 2, (n_groups - Gs) * O * 2);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int a = 0; a < AB; ++a) {
                af[ks][a].u4 = __builtin_amdgcn_raw_buffer_load_b128(rv, (int)a_voff[ks][a], 0, 0);
                ix[ks][a] = __builtin_amdgcn_raw_buffer_load_b16(rm, (int)(a_voff[ks][a] >> 3), 0, 0);
            }
    };

    // ---- dense operand: direct global->LDS loads, swizzled ------------------------------------
    // direct load d (0..DMA_PER_WAVE-1) of this wave fills rows  wave*KT/4 + d*ROWS_PER_DMA + lane/CPR
    // and chunk position lane%CPR, i.e. it must fetch global chunk  (lane%CPR) ^ 4*(row%4).
    constexpr int PHASES = ROWS_PER_DMA >= 4 ? 1 : 4 / ROWS_PER_DMA;
    uint32_t b_src[PHASES];                                    // byte offsets in the stage, by (d*ROWS_PER_DMA)%4 phase
    const int dma_row = lane / CPR, dma_pos = lane % CPR;
#pragma unroll
    for (int ph = 0; ph < PHASES; ++ph) {
        const int row_mod4 = (ph * ROWS_PER_DMA + dma_row) & 3;
        const int64_t col = min(n0 + 8 * (dma_pos ^ (4 * row_mod4)), I - 8);
        b_src[ph] = (uint32_t)(((int64_t)(wave * (KT / 4) + dma_row) * ldh + col) * 2);
    }
    const uint32_t b_row_step = (uint32_t)(ROWS_PER_DMA * ldh * 2);
    auto load_b = [&](int it, int buf) {
        const int64_t t0 = (g_begin + (int64_t)it * 4) * 16;
        const __amdgpu_buffer_rsrc_t rh = rsrc((const char *)h + t0 * ldh * 2, ((T - t0 - 1) * ldh + I) * 2);
#pragma unroll
        for (int d = 0; d < DMA_PER_WAVE; ++d) {
            char *dst = (buf == 0 ? Bs0 : buf == 1 ? Bs1 : Bs2) + (wave * (KT / 4) + d * ROWS_PER_DMA) * (TN * 2);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rh, (lptr_t)dst, 16, (int)(b_src[d % PHASES] + (uint32_t)d * b_row_step), 0, 0, 0);
        }
    };
    auto fetch = [&](int it, int buf, Frag8 (&af)[2][AB], uint32_t (&ix)[2][AB]) {
        load_b(it, buf);
        load_a(it, af, ix);
    };
    // Loads a wave issues per stage; with the fetch of stage s+2 issued before stage s is computed,
    // "stage s+1 has landed" means: at most one stage's worth of this wave's loads still in flight.
    constexpr int LOADS_PER_STAGE = DMA_PER_WAVE + 4 * AB;
    auto next_stage_ready = [&]() {
        wait_vmcnt<LOADS_PER_STAGE>();
        // ... and every other wave's part of it too.  A bare barrier: __syncthreads() would add a
        // workgroup release fence, which the compiler implements by draining every direct-to-LDS
        // load in flight (those of stage s+2 included).  The LDS reads of the stage just computed
        // were drained by the lgkmcnt(0) of its last fragment, so its buffer may be refilled after this.
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };

    // lane's LDS read address pieces for the transposing reads (see the layout note above)
    const int li = lane & 15, q4 = lane >> 4;
    const int rd_row = (8 * (q4 >> 1) + (li >> 2)) * (TN * 2);     // + (32*ks + 16*(j>>1) + 4*(j&1)) rows
    int rd_off[BB];
#pragma unroll
    for (int b = 0; b < BB; ++b)
        rd_off[b] = rd_row + (4 * (((wn * BB + b)) ^ (li >> 2)) + 2 * (q4 & 1) + ((li & 3) >> 1)) * 16 + (li & 1) * 8;

    const uint32_t lds_base[3] = {(uint32_t)(uintptr_t)(lptr_t)Bs0, (uint32_t)(uintptr_t)(lptr_t)Bs1, (uint32_t)(uintptr_t)(lptr_t)Bs2};
    // one stage: the fragment of h for step (ks, b+1) is requested from LDS before the MFMAs of (ks, b) issue
    auto compute = [&](int buf, Frag8 (&af)[2][AB], uint32_t (&ix)[2][AB]) {
        uint32_t addr[BB];
#pragma unroll
        for (int b = 0; b < BB; ++b) addr[b] = lds_base[buf] + (uint32_t)rd_off[b];
        auto read_b = [&](int ks, int b, Frag16 &bf) {
            constexpr int R = TN * 2;
            if (ks == 0) {
                bf.q[0] = lds_read_tr16<0 * R>(addr[b]);  bf.q[1] = lds_read_tr16<4 * R>(addr[b]);
                bf.q[2] = lds_read_tr16<16 * R>(addr[b]); bf.q[3] = lds_read_tr16<20 * R>(addr[b]);
            } else {
                bf.q[0] = lds_read_tr16<32 * R>(addr[b]); bf.q[1] = lds_read_tr16<36 * R>(addr[b]);
                bf.q[2] = lds_read_tr16<48 * R>(addr[b]); bf.q[3] = lds_read_tr16<52 * R>(addr[b]);
            }
        };
        Frag16 bf[2];
        read_b(0, 0, bf[0]);
#pragma unroll
        for (int s = 0; s < 2 * BB; ++s) {
            const int ks = s / BB, b = s % BB;
            const bool last = s + 1 == 2 * BB;
            if (!last) read_b((s + 1) / BB, (s + 1) % BB, bf[(s + 1) & 1]);
#pragma unroll
            for (int a = 0; a < AB; ++a) {
                if (a > 0)     smfmac_32x32x32<0>(acc[a][b], af[ks][a].v, bf[s & 1].v, ix[ks][a]);
                else if (last) smfmac_32x32x32<1>(acc[a][b], af[ks][a].v, bf[s & 1].v, ix[ks][a]);
                else           smfmac_32x32x32<5>(acc[a][b], af[ks][a].v, bf[s & 1].v, ix[ks][a]);
            }
        }
    };

    // Three register sets for the sparse operand and three LDS buffers, rotating by stage: while
    // stage s is computed, the loads of stages s+1 and s+2 are in flight (about two stages of MFMA
    // work, ~2000 cycles, cover the memory latency of a wave that has no sibling on its SIMD).
    // Straight-line loop body, three stages per trip.  Stages past the end of the tensor read as
    // zeros (buffer bounds), so the stage count is padded to a multiple of three with all-zero
    // stages and the fetches that run ahead of the last stage need no guard.  (Split-K slabs other
    // than the last hold a multiple of three stages: see make_plan.)
    Frag8 a0[2][AB], a1[2][AB], a2[2][AB];
    uint32_t i0[2][AB], i1[2][AB], i2[2][AB];
    const int n_trips = (n_iters + 2) / 3;
    if (n_trips > 0) {
        fetch(0, 0, a0, i0);
        fetch(1, 1, a1, i1);
        next_stage_ready();
    }
    for (int tr = 0; tr < n_trips; ++tr) {
        const int it = 3 * tr;
        fetch(it + 2, 2, a2, i2);
        compute(0, a0, i0);
        next_stage_ready();
        fetch(it + 3, 0, a0, i0);
        compute(1, a1, i1);
        next_stage_ready();
        fetch(it + 4, 1, a1, i1);
        compute(2, a2, i2);
        next_stage_ready();
    }

    // ---- epilogue.  The matrix pipeline may still be writing the last accumulators, and the
    // compiler cannot see MFMAs inside asm statements: idle for longer than an 8-pass
    // instruction before the first read of an accumulation register.
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
    for (int a = 0; a < AB; ++a)
#pragma unroll
        for (int b = 0; b < BB; ++b) {
            const int64_t col = n0 + wn * (BB * 32) + b * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = o0 + a * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row < O && col < I) {
                    float *p = out + row * ldo + col;
                    *p = accumulate ? (*p + acc[a][b][r]) : acc[a][b][r];
                }
            }
        }
}

// out[o][i] = (accumulate ? out : 0) + sum_z part[z][o][i], z ascending
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ part, int slabs, int64_t slab_stride,
                                                           float *__restrict__ out, int64_t ldo, int64_t O, int64_t I, int accumulate)
{
    const int64_t n4 = O * (I / 4);
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n4) return;
    const int64_t o = idx / (I / 4), i = (idx % (I / 4)) * 4;
    float4 s = accumulate ? *(const float4 *)(out + o * ldo + i) : make_float4(0.f, 0.f, 0.f, 0.f);
    for (int z = 0; z < slabs; ++z) {
        const float4 v = *(const float4 *)(part + (int64_t)z * slab_stride + o * I + i);
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    *(float4 *)(out + o * ldo + i) = s;
}

// ------------------------------------------------------------------------------------
// host side: tile shape and split-K plan (pure function of the problem size)
// ------------------------------------------------------------------------------------
struct Plan { int shape; int tm, tn; int tiles_m, tiles_n; int slabs; int64_t groups_per_slab; };

static Plan make_plan(int64_t T, int64_t O, int64_t I)
{
    Plan p;
    const int64_t groups = T / 16;
    const int CUS = 256;
    // shape 0: 256x256, shape 1: 128x128, shape 2: 64x256 (few rows)
    if (O <= 64) { p.shape = 2; p.tm = 64; p.tn = 256; }
    else if ((O + 255) / 256 * ((I + 255) / 256) >= CUS) { p.shape = 0; p.tm = 256; p.tn = 256; }
    else { p.shape = 1; p.tm = 128; p.tn = 128; }
    p.tiles_m = (int)((O + p.tm - 1) / p.tm);
    p.tiles_n = (int)((I + p.tn - 1) / p.tn);
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    int slabs = 1;
    if (tiles < CUS && groups >= 64) {
        slabs = (int)((2 * CUS + tiles - 1) / tiles);                 // about two workgroups per CU
        const int64_t max_slabs = groups / 32;                         // at least 512 tokens per slab
        if (slabs > max_slabs) slabs = (int)max_slabs;
        if (slabs < 1) slabs = 1;
    }
    int64_t gps = (groups + slabs - 1) / slabs;
    gps = (gps + 11) / 12 * 12;                                        // whole trips of three LDS stages
    if (gps < 12) gps = 12;
    p.groups_per_slab = gps;
    p.slabs = groups > 0 ? (int)((groups + gps - 1) / gps) : 1;
    return p;
}

size_t update_gemm_smfmac_workspace(int64_t T, int64_t O, int64_t I)
{
    if (T <= 0 || O <= 0 || I <= 0) return 0;
    const Plan p = make_plan(T, O, I);
    return p.slabs > 1 ? (size_t)p.slabs * (size_t)O * (size_t)I * sizeof(float) : 0;
}

hipError_t launch_update_gemm_smfmac(const void *vals, const uint16_t *meta, const void *h, int64_t ldh, float *dW,
                                     int64_t lddw, int64_t T, int64_t O, int64_t I, float beta, void *workspace,
                                     hipStream_t st)
{
    const Plan p = make_plan(T, O, I);
    const int accumulate = beta != 0.f;
    float *out = dW;
    int64_t ldo = lddw, slab_stride = 0;
    int acc_flag = accumulate;
    if (p.slabs > 1) { out = (float *)workspace; ldo = I; slab_stride = O * I; acc_flag = 0; }
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), 1, (unsigned)p.slabs);
#define NM_LAUNCH(WM, WN, AB, BB)                                                                                     \
    hipLaunchKernelGGL((update_gemm_smfmac_kernel<WM, WN, AB, BB>), grid, dim3(256), 0, st, (const uint16_t *)vals,   \
                       meta, (const uint16_t *)h, ldh, out, ldo, slab_stride, T / 16, p.groups_per_slab, O, I,         \
                       p.tiles_m, p.tiles_n, acc_flag)
    if (p.shape == 0) NM_LAUNCH(2, 2, 4, 4);
    else if (p.shape == 1) NM_LAUNCH(2, 2, 2, 2);
    else NM_LAUNCH(1, 4, 2, 2);
#undef NM_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.slabs > 1) {
        const int64_t n4 = O * (I / 4);
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st,
                           (const float *)workspace, p.slabs, slab_stride, dW, lddw, O, I, accumulate);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace nm
