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
// Workgroup = 4 waves (2 x 2), output tile 128 x 128, wave tile 64 x 64 (2 x 2 accumulator blocks).
// The reduction axis advances one 16-token group per stage; the next stage's global loads are issued
// into registers before the current stage's MFMAs.  Split-K over blockIdx.z as in the bf16 kernel.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"

namespace nm {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int F32_TM = 128, F32_TN = 128;
constexpr int F32_LD = 128 + 32;      // LDS row stride in floats: the two half-waves of a fragment read hit disjoint banks

__global__ __launch_bounds__(256) void update_gemm_f32_mfma_kernel(
    const float *__restrict__ vals, const uint16_t *__restrict__ meta, const float *__restrict__ h, int64_t ldh,
    float *__restrict__ out, int64_t ldo, int64_t slab_stride, int64_t n_groups, int64_t groups_per_slab,
    int64_t O, int64_t I, int accumulate)
{
    __shared__ __attribute__((aligned(16))) float As[16 * F32_LD];      // expanded sparse operand: [token in group][o]
    __shared__ __attribute__((aligned(16))) float Bs[16 * F32_LD];      // h rows: [token in group][i]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t o0 = (int64_t)blockIdx.y * F32_TM, i0 = (int64_t)blockIdx.x * F32_TN;
    const int64_t g_begin = (int64_t)blockIdx.z * groups_per_slab;
    const int64_t g_end = min(n_groups, g_begin + groups_per_slab);
    out += (int64_t)blockIdx.z * slab_stride;

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // Threads 0..127 bring the sparse operand (one row of the tile each: 8 kept values + the index word of
    // the group), threads 128..255 bring h (16 rows x 128 columns = 512 float4, four per thread).
    const bool is_a = tid < 128;
    const int64_t o = o0 + tid;                              // (threads of the first half only)
    const bool o_ok = is_a && o < O;
    const int hb = tid - 128;                                // (threads of the second half only)
    float4 pre[4];                                           // A: kept values in pre[0], pre[1]; B: four float4 of h
    uint32_t pre_meta = 0;
    auto prefetch = [&](int64_t G) {
        if (is_a) {
            if (o_ok) {
                const float4 *vp = (const float4 *)(vals + (G * O + o) * 8);
                pre[0] = vp[0]; pre[1] = vp[1];
                pre_meta = meta[G * O + o];
            } else { pre[0] = pre[1] = make_float4(0.f, 0.f, 0.f, 0.f); pre_meta = 0x4444u; }   // positions (0,1) of every quad: zeros
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int idx = hb + 128 * e, r = idx >> 5, c4 = idx & 31;
                const int64_t i = i0 + 4 * c4;
                pre[e] = i < I ? *(const float4 *)(h + (G * 16 + r) * ldh + i) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    };
    auto to_lds = [&]() {
        if (is_a) {
            const float v[8] = {pre[0].x, pre[0].y, pre[0].z, pre[0].w, pre[1].x, pre[1].y, pre[1].z, pre[1].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t nib = (pre_meta >> (4 * q)) & 0xfu, p0 = nib & 3u, p1 = nib >> 2;
#pragma unroll
                for (int p = 0; p < 4; ++p)
                    As[(4 * q + p) * F32_LD + tid] = p0 == (uint32_t)p ? v[2 * q] : (p1 == (uint32_t)p ? v[2 * q + 1] : 0.f);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int idx = hb + 128 * e, r = idx >> 5, c4 = idx & 31;
                *(float4 *)(Bs + r * F32_LD + 4 * c4) = pre[e];
            }
        }
    };

    const int rd = (lane >> 5) * F32_LD + (lane & 31);       // + 2*kk*F32_LD + block offset
    if (g_begin < g_end) prefetch(g_begin);
    for (int64_t G = g_begin; G < g_end; ++G) {
        to_lds();
        __syncthreads();
        if (G + 1 < g_end) prefetch(G + 1);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            float af[2], bf[2];
#pragma unroll
            for (int a = 0; a < 2; ++a) af[a] = As[2 * kk * F32_LD + rd + wm * 64 + a * 32];
#pragma unroll
            for (int b = 0; b < 2; ++b) bf[b] = Bs[2 * kk * F32_LD + rd + wn * 64 + b * 32];
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[a], bf[b], acc[a][b], 0, 0, 0);
        }
        __syncthreads();
    }

#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int64_t col = i0 + wn * 64 + b * 32 + (lane & 31);
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
