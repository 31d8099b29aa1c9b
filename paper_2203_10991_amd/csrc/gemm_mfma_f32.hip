// Update GEMM for binary32 operands on the dense fp32 MFMA path:
//     dW[O x I] (+)= decompress(vals, meta)^T h      (eq. (3)).
//
// gfx950 has sparse matrix instructions for 16-bit and 8-bit operands only, so for NM_F32 the
// compressed operand is expanded to dense rows on its way into LDS (kept values scattered to their
// positions by the index words, zeros elsewhere) and multiplied with v_mfma_f32_32x32x2_f32.  The
// products with the pruned half are executed (as zeros): the format still halves the operand bytes.
//
// Lane layouts of v_mfma_f32_32x32x2_f32 (l = lane): A value of row l%32 for reduction index l/32,
// B value of column l%32 for reduction index l/32, D reg r = row 8*(r/4) + 4*(l/32) + r%4, column l%32.
//
// Workgroup = 4 waves (2 x 2), output tile 128 (rows of dW) x 256 (columns), wave tile 64 x 128 (2 x 4 accumulator
// blocks = 128 accumulator registers).  The tile is wide in the direction of h because expanding the sparse
// operand is vector-ALU work that delays the matrix pipeline of the same SIMD: one expanded row now feeds 256 columns.
// The reduction axis advances one 16-token group per stage through two LDS buffers (one barrier per stage); the
// global loads of the stage after next and the register -> LDS traffic of the next stage are spread between the
// current stage's MFMAs, and the LDS reads of step kk+1 are issued before the MFMAs of step kk.  Every thread
// expands half a row of the sparse operand (two quads) and brings four 16-byte pieces of h.  Split-K over
// blockIdx.z as in the bf16 kernel.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "nm_internal.h"

namespace nm {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int F32_TM = 128, F32_TN = 256;
// LDS row strides in floats: the two half-waves of a fragment read (rows 2kk and 2kk+1) hit disjoint banks
constexpr int F32_LDA = F32_TM + 32, F32_LDB = F32_TN + 32;

// (two workgroups per CU: 128 accumulator registers + at most 128 others per lane)
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void update_gemm_f32_mfma_kernel(
    const float *__restrict__ vals, const uint16_t *__restrict__ meta, const float *__restrict__ h, int64_t ldh,
    float *__restrict__ out, int64_t ldo, int64_t slab_stride, int64_t n_groups, int64_t groups_per_slab,
    int64_t O, int64_t I, int accumulate)
{
    __shared__ __attribute__((aligned(16))) float As2[2][16 * F32_LDA];  // expanded sparse operand: [token in group][o]
    __shared__ __attribute__((aligned(16))) float Bs2[2][16 * F32_LDB];  // h rows: [token in group][i]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t o0 = (int64_t)blockIdx.y * F32_TM, i0 = (int64_t)blockIdx.x * F32_TN;
    const int64_t g_begin = (int64_t)blockIdx.z * groups_per_slab;
    const int64_t g_end = min(n_groups, g_begin + groups_per_slab);
    out += (int64_t)blockIdx.z * slab_stride;

    f32x16 acc[2][4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // sparse operand: thread = row ar of the tile, half ah of the group (quads 2ah, 2ah+1: kept values 4ah..4ah+3,
    // index bits 8ah..8ah+7).  h: 16 rows x 256 columns = 1024 pieces of 16 bytes, four per thread.
    const int ar = tid & 127, ah = tid >> 7;
    // Rows >= O and columns >= I are clamped to the last valid ones (no branch in the loop): what they
    // contribute lands in outputs that are never stored.
    const int64_t o = min(o0 + ar, O - 1);
    const float *a_src = vals + o * 8 + 4 * ah;
    const uint16_t *m_src = meta + o;
    auto b_ptr = [&](int e) {
        const int idx = tid + 256 * e, r = idx >> 6, c4 = idx & 63;
        return h + (int64_t)r * ldh + min(i0 + 4 * c4, I - 4);
    };
    const float *b_src0 = b_ptr(0), *b_src1 = b_ptr(1), *b_src2 = b_ptr(2), *b_src3 = b_ptr(3);
    // One stage's share of this thread on its way from global memory to LDS.  Two of them alternate, so a load has a
    // whole stage (about two microseconds) to arrive.  (Separate members, no arrays: arrays here end up in LDS.)
    struct Pre { float4 a, b0, b1, b2, b3; uint32_t meta; };
    Pre pre_x, pre_y;
    auto prefetch = [&](int64_t G, Pre &pre) {
        pre.a = *(const float4 *)(a_src + G * O * 8);
        pre.meta = (uint32_t)m_src[G * O] >> (8 * ah);
        const int64_t step = G * 16 * ldh;
        pre.b0 = *(const float4 *)(b_src0 + step);
        pre.b1 = *(const float4 *)(b_src1 + step);
        pre.b2 = *(const float4 *)(b_src2 + step);
        pre.b3 = *(const float4 *)(b_src3 + step);
    };
    const int b_dst = (tid >> 6) * F32_LDB + 4 * (tid & 63);            // piece e lands 4 rows further down per e
    // registers -> LDS in four pieces, so that the loop can spread them between its MFMAs:
    // piece c = quad c of this thread's half row (c < 2) and h piece c
    auto lds_piece = [&](int c, int buf, const Pre &pre) {
        float *As = As2[buf], *Bs = Bs2[buf];
        if (c < 2) {
            // quad c of the half row: zeros to its four tokens, then the two kept values on top at the positions the
            // index bits name (LDS executes a wave's writes in order); far fewer vector-ALU instructions than
            // selecting each of the four values
            const float v0 = c == 0 ? pre.a.x : pre.a.z, v1 = c == 0 ? pre.a.y : pre.a.w;
            const uint32_t p0 = (pre.meta >> (4 * c)) & 3u, p1 = (pre.meta >> (4 * c + 2)) & 3u;
            float *q = As + (8 * ah + 4 * c) * F32_LDA + ar;
#pragma unroll
            for (int p = 0; p < 4; ++p) q[p * F32_LDA] = 0.f;
            q[p0 * F32_LDA] = v0;
            q[p1 * F32_LDA] = v1;
        }
        const float4 piece = c == 0 ? pre.b0 : c == 1 ? pre.b1 : c == 2 ? pre.b2 : pre.b3;
        *(float4 *)(Bs + b_dst + 4 * c * F32_LDB) = piece;
    };

    const int rd_a = (lane >> 5) * F32_LDA + (lane & 31) + wm * 64;      // + 2*kk*F32_LDA + 32*a
    const int rd_b = (lane >> 5) * F32_LDB + (lane & 31) + wn * 128;     // + 2*kk*F32_LDB + 32*b
    float af[2][2], bf[2][4];                            // operand registers in two sets
    auto read_step = [&](int buf, int kk, int set) {
        const float *As = As2[buf], *Bs = Bs2[buf];
#pragma unroll
        for (int a = 0; a < 2; ++a) af[set][a] = As[2 * kk * F32_LDA + rd_a + a * 32];
#pragma unroll
        for (int b = 0; b < 4; ++b) bf[set][b] = Bs[2 * kk * F32_LDB + rd_b + b * 32];
    };
    // One stage: multiplies the group in LDS buffer `cur`; `next` holds the following group (loaded a stage ago) and
    // goes to the other buffer; `after` receives the loads of the group after that.
    // Step kk: the LDS reads of step kk+1 first (in step 7: those of the next stage's step 0), then the eight MFMAs.
    // Behind the first two MFMAs of step 0 go the global loads, behind those of steps 1..4 one piece each of the next
    // stage: vector-ALU and memory instructions issue while the matrix pipeline works on the MFMAs already issued.
    // The stage's one barrier sits after step 6: by then this wave has written its pieces of the next stage and holds
    // the operands of step 7 in registers, so past the barrier the next stage may be read and -- from its step 1
    // on -- the buffer of this stage overwritten.
    auto stage = [&](int64_t G, auto cur_c, const Pre &next, Pre &after) {
        constexpr int cur = decltype(cur_c)::value;
        // No branches in here: a branch makes the compiler merge its counts of outstanding LDS operations at the join,
        // and the merged count makes the MFMAs behind it wait for the reads and writes just issued.  At the end of
        // the slab the pieces, the reads of "the next stage" and the loads (of the last group again) are done all
        // the same and nobody uses them.
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            if (kk + 1 < 8) read_step(cur, kk + 1, (kk + 1) & 1);
            else read_step(cur ^ 1, 0, 0);
            __builtin_amdgcn_sched_barrier(0);           // (keeps the reads ahead of the MFMAs: the scheduler would sink them)
#pragma unroll
            for (int b = 0; b < 2; ++b)
                acc[0][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[kk & 1][0], bf[kk & 1][b], acc[0][b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (kk == 0) prefetch(min(G + 2, g_end - 1), after);
            if (kk >= 1 && kk <= 4) lds_piece(kk - 1, cur ^ 1, next);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 2; b < 4; ++b)
                acc[0][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[kk & 1][0], bf[kk & 1][b], acc[0][b], 0, 0, 0);
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc[1][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[kk & 1][1], bf[kk & 1][b], acc[1][b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (kk == 6) {
                // orders LDS traffic only: the global loads in flight stay in flight (__syncthreads() would wait for them)
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    if (g_begin < g_end) {
        prefetch(g_begin, pre_x);
#pragma unroll
        for (int c = 0; c < 4; ++c) lds_piece(c, 0, pre_x);
        if (g_begin + 1 < g_end) prefetch(g_begin + 1, pre_y);
        __syncthreads();
        read_step(0, 0, 0);
    }
    for (int64_t G = g_begin; G < g_end; G += 2) {
        stage(G, std::integral_constant<int, 0>{}, pre_y, pre_x);
        if (G + 1 < g_end) stage(G + 1, std::integral_constant<int, 1>{}, pre_x, pre_y);
    }

#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int64_t col = i0 + wn * 128 + b * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = o0 + wm * 64 + a * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row < O && col < I) {
                    float *p = out + row * ldo + col;
                    *p = accumulate ? (*p + acc[a][b][r]) : acc[a][b][r];
                }
            }
        }
}

// split-K plan: a pure function of the problem size
struct PlanF32 { int tiles_m, tiles_n, slabs; int64_t groups_per_slab; };
static PlanF32 make_plan_f32(int64_t T, int64_t O, int64_t I)
{
    PlanF32 p;
    const int64_t groups = T / 16;
    p.tiles_m = (int)((O + F32_TM - 1) / F32_TM);
    p.tiles_n = (int)((I + F32_TN - 1) / F32_TN);
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    int64_t slabs = 1;
    if (tiles < 256 && groups >= 16) {
        slabs = (2 * 256 + tiles - 1) / tiles;            // about two workgroups per CU
        if (slabs > groups / 8) slabs = groups / 8;       // at least 128 tokens per slab
        if (slabs < 1) slabs = 1;
    }
    p.groups_per_slab = groups > 0 ? (groups + slabs - 1) / slabs : 1;
    p.slabs = groups > 0 ? (int)((groups + p.groups_per_slab - 1) / p.groups_per_slab) : 1;
    return p;
}

size_t update_gemm_f32_workspace(int64_t T, int64_t O, int64_t I)
{
    if (T <= 0 || O <= 0 || I <= 0) return 0;
    const PlanF32 p = make_plan_f32(T, O, I);
    return p.slabs > 1 ? (size_t)p.slabs * (size_t)O * (size_t)I * sizeof(float) : 0;
}

hipError_t launch_update_gemm_f32(const void *vals, const uint16_t *meta, const void *h, int64_t ldh, float *dW,
                                  int64_t lddw, int64_t T, int64_t O, int64_t I, float beta, void *workspace,
                                  hipStream_t st)
{
    if (O == 0 || I == 0) return hipSuccess;
    const PlanF32 p = make_plan_f32(T, O, I);
    const int accumulate = beta != 0.f;
    float *out = dW;
    int64_t ldo = lddw, slab_stride = 0;
    int acc_flag = accumulate;
    if (p.slabs > 1) { out = (float *)workspace; ldo = I; slab_stride = O * I; acc_flag = 0; }
    dim3 grid((unsigned)p.tiles_n, (unsigned)p.tiles_m, (unsigned)p.slabs);
    hipLaunchKernelGGL(update_gemm_f32_mfma_kernel, grid, dim3(256), 0, st, (const float *)vals, meta, (const float *)h,
                       ldh, out, ldo, slab_stride, T / 16, p.groups_per_slab, O, I, acc_flag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.slabs > 1) e = launch_splitk_reduce((const float *)workspace, p.slabs, dW, lddw, O, I, accumulate, 1.0f, st);
    return e;
}

}  // namespace nm
