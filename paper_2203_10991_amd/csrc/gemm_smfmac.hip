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
// stage, double buffered, one barrier per stage.  Split-K over blockIdx.z writes binary32
// partials that a second kernel sums in a fixed order (deterministic; no atomics).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"

namespace nm {

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int KT = 64;            // tokens per LDS stage (two 32-token MFMA steps)
constexpr int LDS_PAD = 32;       // bf16 elements of row padding: row stride = 16 banks mod 64

union Frag16 { bf16x16 v; s16x4 q[4]; };
union Frag8 { bf16x8 v; uint4 u; };

template <int WM, int WN, int AB, int BB>
__global__ __launch_bounds__(256) void update_gemm_smfmac_kernel(
    const uint16_t *__restrict__ vals, const uint16_t *__restrict__ meta, const uint16_t *__restrict__ h, int64_t ldh,
    float *__restrict__ out, int64_t ldo, int64_t slab_stride,       // out + z*slab_stride
    int64_t n_groups, int64_t groups_per_slab, int64_t O, int64_t I, int tiles_m, int tiles_n, int accumulate)
{
    constexpr int TM = WM * AB * 32, TN = WN * BB * 32;
    constexpr int RS = TN + LDS_PAD;                     // LDS row stride in elements
    constexpr int CHUNKS_PER_ROW = TN / 8;
    constexpr int CHUNKS_PER_THREAD = KT * CHUNKS_PER_ROW / 256;
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][KT * RS];

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

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
        for (int b = 0; b < BB; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    const int n_iters = (int)((g_end - g_begin + 3) / 4);      // 4 token groups per stage

    // ---- operand fetch helpers -------------------------------------------------------------
    const int kg = lane >> 5;                                  // which 16-token group of a 32-token step
    Frag8 a_cur[2][AB], a_nxt[2][AB];
    uint32_t idx_cur[AB], idx_nxt[AB];
    uint4 stage[CHUNKS_PER_THREAD];

    auto load_a = [&](int it, Frag8 (&af)[2][AB], uint32_t (&ix)[AB]) {
#pragma unroll
        for (int a = 0; a < AB; ++a) {
            const int64_t o = o0 + a * 32 + (lane & 31);
            uint32_t m01[2];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const int64_t G = g_begin + (int64_t)it * 4 + 2 * ks + kg;
                const bool ok = (G < g_end) & (o < O);
                const int64_t e = ok ? (G * O + o) : 0;
                uint4 v = *(const uint4 *)(vals + e * 8);
                uint32_t m = meta[e];
                if (!ok) { v = make_uint4(0, 0, 0, 0); m = 0x4444u; }
                af[ks][a].u = v;
                m01[ks] = m;
            }
            ix[a] = m01[0] | (m01[1] << 16);
        }
    };
    auto load_b = [&](int it) {
#pragma unroll
        for (int p = 0; p < CHUNKS_PER_THREAD; ++p) {
            const int c = tid + 256 * p, row = c / CHUNKS_PER_ROW, cc = c % CHUNKS_PER_ROW;
            const int64_t t = (g_begin + (int64_t)it * 4) * 16 + row;
            const int64_t col = n0 + cc * 8;
            const bool ok = (t < g_end * 16) & (col < I);
            stage[p] = ok ? *(const uint4 *)(h + t * ldh + col) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_b = [&](int buf) {
#pragma unroll
        for (int p = 0; p < CHUNKS_PER_THREAD; ++p) {
            const int c = tid + 256 * p, row = c / CHUNKS_PER_ROW, cc = c % CHUNKS_PER_ROW;
            *(uint4 *)(&Bs[buf][row * RS + cc * 8]) = stage[p];
        }
    };

    // lane's LDS read offsets (elements) for the transposing reads
    const int li = lane & 15, q = lane >> 4;
    const int b_row0 = 8 * (q >> 1) + (li >> 2);                // + 32*ks + 16*(j>>1) + 4*(j&1)
    const int b_col0 = wn * (BB * 32) + 16 * (q & 1) + 4 * (li & 3);   // + 32*bn

    if (n_iters > 0) {
        load_a(0, a_cur, idx_cur);
        load_b(0);
        store_b(0);
    }
    __syncthreads();

    for (int it = 0; it < n_iters; ++it) {
        const int buf = it & 1;
        const bool more = it + 1 < n_iters;
        if (more) {
            load_b(it + 1);
            load_a(it + 1, a_nxt, idx_nxt);
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int b = 0; b < BB; ++b) {
                Frag16 bf;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int row = 32 * ks + 16 * (j >> 1) + 4 * (j & 1) + b_row0;
                    const int col = 32 * b + b_col0;
                    bf.q[j] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) s16x4 *)(&Bs[buf][row * RS + col]));
                }
#pragma unroll
                for (int a = 0; a < AB; ++a) {
                    if (ks == 0)
                        acc[a][b] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a_cur[0][a].v, bf.v, acc[a][b], (int)idx_cur[a], 0, 0);
                    else
                        acc[a][b] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a_cur[1][a].v, bf.v, acc[a][b], (int)idx_cur[a], 0, 1);
                }
            }
        }
        if (more) {
            store_b(buf ^ 1);
#pragma unroll
            for (int a = 0; a < AB; ++a) {
                a_cur[0][a] = a_nxt[0][a];
                a_cur[1][a] = a_nxt[1][a];
                idx_cur[a] = idx_nxt[a];
            }
        }
        __syncthreads();
    }

    // ---- epilogue
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
    gps = (gps + 3) / 4 * 4;                                           // whole LDS stages
    if (gps < 4) gps = 4;
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
