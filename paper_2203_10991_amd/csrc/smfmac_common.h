// Device helpers shared by the sparse-MFMA update-GEMM kernels (16-bit and 8-bit operands): compile-time loops,
// asm-defined accumulator blocks, LDS reads issued as asm, explicit wait counts, the workgroup -> tile map.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "nm_internal.h"     // AlphaArg

namespace nm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));


union Frag16 { bf16x16 v; s16x4 q[4]; };
union Frag8 { bf16x8 v; u32x4 u4; };

typedef __attribute__((address_space(3))) void *lptr_t;

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>)
template <typename F, int... Is> __device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F> __device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// The accumulator blocks of a wave must own the accumulation-register half (AGPRs) of the
// register file for the whole kernel, with everything else in VGPRs.  Left to itself the compiler
// keeps accumulators in VGPRs and shuffles blocks to and from AGPRs around every MFMA, so each
// definition of an accumulator is an asm statement with an AGPR operand:
//   acc_zero   D = 0*0 + 0 with a dense MFMA (inline-constant C): writes 16 AGPRs at once
//   smfmac     D += A(4:2 sparse, index word in the low half of idx) * B, optionally preceded by
//              a wait until at most LGKM LDS reads are outstanding (LGKM < 0: no wait); ABID picks the
//              half of idx that holds the index word
// IN_VGPR: the block lives in ordinary registers instead (the compiler splits a wave's register budget evenly
// between the two halves of the file, so a kernel with more than 128 accumulation registers per wave at two waves
// per SIMD keeps the excess there).
template <bool IN_VGPR = false>
__device__ __forceinline__ void acc_zero(f32x16 &acc)
{
    const bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    // (the compiler does not know this asm is an MFMA: keep the required distance from the VALU moves that write z)
    if constexpr (IN_VGPR) asm volatile("s_nop 4\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %1, 0" : "=v"(acc) : "v"(z));
    else                   asm volatile("s_nop 4\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %1, 0" : "=a"(acc) : "v"(z));
}
template <int LGKM, int ABID, bool IN_VGPR = false>
__device__ __forceinline__ void smfmac_32x32x32(f32x16 &acc, const bf16x8 &a, const bf16x16 &b, uint32_t idx)
{
    if constexpr (LGKM >= 0) asm volatile("s_waitcnt lgkmcnt(%0)" : : "n"(LGKM));
    if constexpr (IN_VGPR) {
        if constexpr (ABID == 0)
            asm volatile("v_smfmac_f32_32x32x32_bf16 %0, %1, %2, %3" : "+v"(acc) : "v"(a), "v"(b), "v"(idx));
        else
            asm volatile("v_smfmac_f32_32x32x32_bf16 %0, %1, %2, %3 abid:1" : "+v"(acc) : "v"(a), "v"(b), "v"(idx));
    } else {
        if constexpr (ABID == 0)
            asm volatile("v_smfmac_f32_32x32x32_bf16 %0, %1, %2, %3" : "+a"(acc) : "v"(a), "v"(b), "v"(idx));
        else
            asm volatile("v_smfmac_f32_32x32x32_bf16 %0, %1, %2, %3 abid:1" : "+a"(acc) : "v"(a), "v"(b), "v"(idx));
    }
}

// An empty statement that "rewrites" an accumulator block: placed after the idle cycles that follow the last MFMA,
// it makes everything that reads the block later (stores, or copies the compiler makes for them) depend on it, so
// that none of it can be placed above the wait.  (The compiler cannot see that the asm MFMAs are still in flight.)
template <bool IN_VGPR = false>
__device__ __forceinline__ void acc_settled(f32x16 &acc)
{
    if constexpr (IN_VGPR) asm volatile("" : "+v"(acc));
    else                   asm volatile("" : "+a"(acc));
}

// One accumulator element to global memory, straight from the register it lives in (memory instructions take
// accumulation registers as data): otherwise the compiler copies whole blocks to ordinary registers first and,
// short of those, spills accumulators to scratch around the epilogue.
template <bool IN_VGPR = false>
__device__ __forceinline__ void store_acc(float *p, float v)
{
    if constexpr (IN_VGPR) asm volatile("global_store_dword %0, %1, off" : : "v"(p), "v"(v) : "memory");
    else                   asm volatile("global_store_dword %0, %1, off" : : "v"(p), "a"(v) : "memory");
}

// LDS reads are issued as asm so that the compiler does not order them against the direct
// global->LDS loads still in flight for later stages; that ordering is explicit (vmcnt wait +
// barrier per stage), and so are the waits for the reads themselves (LGKM above).
template <int OFFSET> __device__ __forceinline__ s16x4 lds_read_tr16(uint32_t addr)     // 4 tokens x 16 columns transposed per 16 lanes
{
    s16x4 r;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFFSET) : "memory");
    return r;
}
template <int OFFSET> __device__ __forceinline__ u32x4 lds_read_b128(uint32_t addr)
{
    u32x4 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFFSET) : "memory");
    return r;
}
template <int OFFSET> __device__ __forceinline__ uint32_t lds_read_b32(uint32_t addr)
{
    uint32_t r;
    asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFFSET) : "memory");
    return r;
}
// refill forms: the destination is the register the previous value of the same fragment lives in (read-write operand),
// so a fragment keeps its registers for the whole kernel
template <int OFFSET> __device__ __forceinline__ void lds_refill_tr16(s16x4 &r, uint32_t addr)
{
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "+v"(r) : "v"(addr), "n"(OFFSET) : "memory");
}
template <int OFFSET> __device__ __forceinline__ void lds_refill_b128(u32x4 &r, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "+v"(r) : "v"(addr), "n"(OFFSET) : "memory");
}
template <int OFFSET> __device__ __forceinline__ void lds_refill_b32(uint32_t &r, uint32_t addr)
{
    asm volatile("ds_read_b32 %0, %1 offset:%2" : "+v"(r) : "v"(addr), "n"(OFFSET) : "memory");
}
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
template <int OFFSET> __device__ __forceinline__ u32x2 lds_read_b64(uint32_t addr)
{
    u32x2 r;
    asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFFSET) : "memory");
    return r;
}

// s_waitcnt vmcnt(N) only (expcnt / lgkmcnt left at their maxima): at most N vector-memory loads still in flight
template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// ---- tile assignment.  Workgroups are dealt round-robin to the 8 XCDs (workgroup id % 8), 32 CUs and one
// L2 each; the 32 tiles resident on an XCD form a block of 8 M-tiles x 4 N-tiles (N fastest), so that
// they share operand strips inside its L2 from the first stage on (8 vals strips + 4 h strips feed 32 tiles).
// Preferred map, when both tile counts are multiples of 16: the XCDs form a 2 x 4 grid and the whole GPU
// works on one 16 x 16 block of tiles at a time.  Of all 8-XCD arrangements this one streams the fewest
// bytes per block from HBM (16 vals strips + 16 h strips); strips shared between XCDs meet in the
// memory-side cache.  Otherwise: one band of M-tiles at a time, XCD x owning the N-tiles [x*nx, (x+1)*nx).
__device__ __forceinline__ void tile_of_workgroup(int bid_, int tiles_m, int tiles_n, int &tm, int &tn)
{
    if (tiles_m % 16 == 0 && tiles_n % 16 == 0) {
        const int bid = bid_, xcd = bid % 8, slot = bid / 8;         // slot: this XCD's running tile count
        const int round = slot / 32, local = slot % 32, bands = tiles_m / 16;
        tm = (round % bands) * 16 + (xcd / 4) * 8 + local / 4;
        tn = (round / bands) * 16 + (xcd % 4) * 4 + local % 4;
    } else {
        const int n_tiles = tiles_m * tiles_n, bid = bid_;
        const int nx = tiles_n / 8;                                    // N-tiles per XCD
        if (tiles_n % 8 == 0 && nx <= 32) {
            const int band_rows = 32 / nx > 0 ? 32 / nx : 1;           // M-tiles per band: band_rows * nx ~ 32 CUs
            const int xcd = bid % 8, slot = bid / 8;                   // slot: this XCD's running tile count
            const int per_band = band_rows * nx;
            const int band = slot / per_band, local = slot % per_band;
            // the last band may be short: its slots are re-dealt over the rows it has (per XCD the band then holds
            // fewer tiles, and every slot still belongs to exactly one tile)
            const int full_bands = tiles_m / band_rows;
            // N-tile index fastest: tiles that share an h strip AND tiles that share a vals strip start within a few
            // dispatches of each other, so both kinds of sharing are live in the L2 from the first stage on
            if (band < full_bands) { tm = band * band_rows + local / nx; tn = xcd * nx + local % nx; }
            else {
                const int l2 = slot - full_bands * per_band;            // index inside the short band
                tm = full_bands * band_rows + l2 / nx; tn = xcd * nx + l2 % nx;
            }
        } else {
            // fallback: contiguous run of tiles per XCD when the count divides evenly, N-fastest inside bands of 8 M-tiles
            int t = bid;
            if (n_tiles % 8 == 0) t = (bid % 8) * (n_tiles / 8) + bid / 8;
            constexpr int BAND = 8;
            const int band = t / (BAND * tiles_n);
            const int band_rows = min(BAND, tiles_m - band * BAND);
            const int in_band = t - band * BAND * tiles_n;
            tm = band * BAND + in_band % band_rows;
            tn = in_band / band_rows;
        }
    }
}

// the output scale of a kernel: a host value, or that value times two inverse scales read from device memory
__device__ __forceinline__ float alpha_of(const AlphaArg &al)
{
    return al.inv_a ? al.value * al.inv_a[1] * al.inv_b[1] : al.value;
}

// The dense operand as row-shifted views of one [rows x cb] matrix (a convolution's im2col matrix that is never
// materialised): column block j of h is x read rows[j] rows further down, h[t][j*cb + c] = x[(t + rows[j])*ldh + c];
// rows -margin .. T+margin-1 of x are readable.
struct ShiftArg { int cb, n, margin; int rows[32]; };

// Split-K launches (gridDim.z slabs of the reduction axis, gridDim.x tiles): workgroups are dealt round-robin to the
// XCDs in launch order (x fastest, then z).  With a tile count that is a multiple of 8 a tile stays on one XCD for
// every slab and the single-pass tile map (compact tile sets per XCD) is still right.  Otherwise the tiles of one
// slab would land on all eight XCDs, each pulling every slab's rows of both operands through the fabric; the
// (slab, tile) pairs are then re-dealt: XCD x takes a contiguous run of the slab-major list, i.e. whole slabs (a
// slab straddles at most two XCDs), whose tiles share the slab's rows through that XCD's L2.
__device__ __forceinline__ void tile_and_slab_of_workgroup(int tiles_m, int tiles_n, int &tm, int &tn, int &slab)
{
    if (gridDim.z > 1 && gridDim.x % 8 != 0) {
        const unsigned n = gridDim.x * gridDim.z;
        const unsigned L = blockIdx.z * gridDim.x + blockIdx.x, xcd = L % 8, idx = L / 8;
        const unsigned first = xcd * (n / 8) + min(xcd, n % 8);        // workgroups that XCDs 0 .. xcd-1 hold
        const unsigned g = first + idx;
        slab = (int)(g / gridDim.x);
        const int t = (int)(g % gridDim.x);
        tm = t / tiles_n; tn = t % tiles_n;
    } else {
        slab = (int)blockIdx.z;
        tile_of_workgroup((int)blockIdx.x, tiles_m, tiles_n, tm, tn);
    }
}

}  // namespace nm
