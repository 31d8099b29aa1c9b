// Sanitizer driver for the host side of the C ABI (test infrastructure): csrc/nm_abi.hip is compiled for the host
// only under -fsanitize=address,undefined and linked with the stub launchers below instead of the kernels, so the
// argument validation -- everything that runs before a launch -- executes on a machine without a GPU.  The driver
// walks the error paths (null, ragged, misaligned, overlapping, absurdly large arguments: the range arithmetic must
// not overflow) and the accepting paths (on which the stubs read what the real launchers read on the host).
// Run by tests/test_sanitizers.py.  Exit status 0 = every call returned what it should and no sanitizer reported.
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "nm_mvue.h"

static int g_launches = 0;
namespace nm {
struct AlphaArg { float value; const float *inv_a, *inv_b; };      // layout of the library's own (passed by value)
hipError_t launch_prune(int, int, int, const void *, int64_t, int64_t, int64_t, uint64_t, uint32_t, void *, uint16_t *, void *, int64_t,
                        hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_prune_producer(int, int, int, const void *, int64_t, const void *, int64_t, int64_t, int64_t, uint64_t, uint32_t, void *,
                                 int64_t, void *, uint16_t *, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_prune_transposed(int, int, const void *, int64_t, int64_t, int64_t, uint64_t, uint32_t, void *, uint16_t *,
                                   hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_prune_4of8_approx(int, const void *, int64_t, int64_t, int64_t, uint64_t, uint32_t, void *, uint32_t *, void *, int64_t,
                                    hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_compress(int, int, const void *, int64_t, int64_t, int64_t, void *, uint16_t *, int32_t *, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_prune_q8(int, int, const void *, int64_t, int64_t, int64_t, uint64_t, uint32_t, float, const float *, uint8_t *, uint32_t *,
                           hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_prune_q8_transposed(int, int, const void *, int64_t, int64_t, int64_t, uint64_t, uint32_t, float, const float *, uint8_t *,
                                      uint32_t *, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_q8_scale(int, const void *, int64_t, int64_t, int64_t, float, float *, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_cast_e4m3(int, const void *, int64_t, int64_t, int64_t, const float *, uint8_t *, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_rw_mix_probe(const void *, void *, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_update_gemm(int, const void *, const uint16_t *, const void *, int64_t, float *, int64_t, int64_t, int64_t, int64_t, float,
                              void *, size_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_update_gemm_q8(const uint8_t *, const uint32_t *, const uint8_t *, int64_t, float *, int64_t, int64_t, int64_t, int64_t,
                                 AlphaArg, float, void *, hipStream_t) { ++g_launches; return hipSuccess; }
static int64_t read_rows(const int64_t *rows, int n) { int64_t s = 0; for (int j = 0; j < n; ++j) s += rows[j]; return s; }
hipError_t launch_update_gemm_smfmac_shifted(const void *, const uint16_t *, const void *, int64_t, int64_t, const int64_t *rows, int n, float *,
                                             int64_t, int64_t, int64_t, float, void *, hipStream_t)
{ ++g_launches; return read_rows(rows, n) == INT64_MIN ? hipErrorUnknown : hipSuccess; }
hipError_t launch_update_gemm_q8_shifted(const uint8_t *, const uint32_t *, const uint8_t *, int64_t, int64_t, const int64_t *rows, int n,
                                         float *, int64_t, int64_t, int64_t, AlphaArg, float, void *, hipStream_t)
{ ++g_launches; return read_rows(rows, n) == INT64_MIN ? hipErrorUnknown : hipSuccess; }
// split-K whenever there are few output tiles, as the real plans do (sizes only matter to the checks)
size_t update_gemm_workspace(int, int64_t T, int64_t O, int64_t I) { return O * I <= 1 << 20 && T >= 1024 ? (size_t)(2 * O * I * 4) : 0; }
size_t update_gemm_q8_workspace(int64_t T, int64_t O, int64_t I) { return update_gemm_workspace(1, T, O, I); }
size_t update_gemm_smfmac_shifted_workspace(int64_t T, int64_t O, int64_t I) { return update_gemm_workspace(1, T, O, I); }
size_t update_gemm_q8_shifted_workspace(int64_t T, int64_t O, int64_t I) { return update_gemm_workspace(1, T, O, I); }
size_t static_scratch_bytes() { return (size_t)32 << 20; }
static char fake_scratch[64];
hipError_t static_scratch(void **p) { *p = fake_scratch; return hipSuccess; }
}  // namespace nm

static int failures = 0;
#define EXPECT(call, code)                                                                                  \
    do {                                                                                                    \
        const int before_ = g_launches;                                                                     \
        const int rc_ = (call);                                                                             \
        if (rc_ != (code)) { fprintf(stderr, "line %d: %s -> %d (%s), wanted %d\n", __LINE__, #call, rc_, nm_last_error(), (int)(code)); ++failures; } \
        if ((code) != 0 && g_launches != before_) { fprintf(stderr, "line %d: launched despite error\n", __LINE__); ++failures; } \
        if ((code) != 0 && !nm_last_error()[0]) { fprintf(stderr, "line %d: no message\n", __LINE__); ++failures; }   \
    } while (0)

int main()
{
    // "device" buffers: host memory of exactly the size the shapes need (never dereferenced by the ABI), 16-byte aligned
    const int64_t T = 1024, O = 64, I = 128;
    std::vector<uint8_t> gbuf(T * O * 4 + 64), vbuf(T / 2 * O * 4 + 64), mbuf(T / 16 * O * 4 + 64), hbuf(T * I * 4 + 64),
        dbuf(T * O * 4 + 64), wbuf(O * I * 4 + 64), wsbuf(2 * O * 144 * 4 + 64), xbuf((T + 64) * I * 2 + 64);
    auto al = [](std::vector<uint8_t> &v) { return (void *)(((uintptr_t)v.data() + 15) & ~(uintptr_t)15); };
    void *g = al(gbuf), *vals = al(vbuf), *meta = al(mbuf), *h = al(hbuf), *dense = al(dbuf), *ws = al(wsbuf), *x = al(xbuf);
    float *dW = (float *)al(wbuf);
    uint16_t *m16 = (uint16_t *)meta;
    uint32_t *m32 = (uint32_t *)meta;
    const size_t wsb = 2 * O * I * 4, wsb_conv = 2 * O * 144 * 4;
    const int64_t huge = (int64_t)1 << 61;

    // ---- accepting paths
    for (int dt = 0; dt < 2; ++dt) {
        EXPECT(mvue_prune_1of2(g, T, O, O, dt, 1, 2, vals, m16, dense, O, nullptr), NM_OK);
        EXPECT(mvue_prune_2of4(g, T, O, O, dt, 1, 2, 0, vals, m16, nullptr, 0, nullptr), NM_OK);
        EXPECT(mvue_prune_2of4(g, T, O, O, dt, 1, 2, 1, vals, m16, dense, O, nullptr), NM_OK);
        EXPECT(mvue_prune_1of4(g, T, O, O, dt, 1, 2, vals, m16, dense, O, nullptr), NM_OK);
        EXPECT(mvue_prune_4of8_approx(g, T, O, O, dt, 1, 2, vals, m32, dense, O, nullptr), NM_OK);
        EXPECT(nm_prune_greedy(g, T, O, O, dt, 2, 4, vals, m16, dense, O, nullptr), NM_OK);
        EXPECT(nm_prune_greedy(g, T, O, O, dt, 1, 2, vals, m16, nullptr, 0, nullptr), NM_OK);
        EXPECT(mvue_prune_2of4_t(g, T, O, T, dt, 1, 2, 0, vals, m16, nullptr), NM_OK);
        EXPECT(mvue_prune_1of2_t(g, T, O, T, dt, 1, 2, vals, m16, nullptr), NM_OK);
        EXPECT(nm_compress(dense, T, O, O, dt, 2, 4, vals, m16, nullptr, nullptr), NM_OK);
        EXPECT(mvue_prune_2of4_q8(g, T, O, O, dt, 1, 2, 0, 0.5f, (uint8_t *)vals, m32, nullptr), NM_OK);
        EXPECT(mvue_prune_1of2_q8(g, T, O, O, dt, 1, 2, 0.5f, (uint8_t *)vals, m32, nullptr), NM_OK);
        EXPECT(mvue_prune_2of4_q8_t(g, T, O, T, dt, 1, 2, 1, 0.5f, nullptr, (uint8_t *)vals, m32, nullptr), NM_OK);
        EXPECT(mvue_prune_1of2_q8_t(g, T, O, T, dt, 1, 2, 0.5f, nullptr, (uint8_t *)vals, m32, nullptr), NM_OK);
        EXPECT(nm_update_gemm(vals, m16, h, I, dW, I, T, O, I, dt, 0.f, ws, wsb, nullptr), NM_OK);
        EXPECT(nm_update_gemm_static(vals, m16, h, I, dW, I, T, O, I, dt, 1.f, nullptr), NM_OK);
    }
    EXPECT(nm_update_gemm(vals, m16, h, I, dW, I, T, O, I, NM_F32_BF16X3, 0.f, ws, wsb, nullptr), NM_OK);
    EXPECT(nm_update_gemm_q8((const uint8_t *)vals, m32, (const uint8_t *)h, I, dW, I, T, O, I, 1.f, 0.f, ws, wsb, nullptr), NM_OK);
    const int64_t shifts[9] = {-7, -6, -5, -1, 0, 1, 5, 6, 7};
    const int64_t cb = 16;
    void *x0 = (char *)x + 16 * cb * 2;             // row 0 with 16 margin rows before it
    EXPECT(nm_update_gemm_shifted(vals, m16, x0, cb, cb, shifts, 9, dW, 9 * cb, T, O, NM_BF16, 0.f, ws, wsb_conv, nullptr), NM_OK);
    EXPECT(nm_update_gemm_q8_shifted((const uint8_t *)vals, m32, (const uint8_t *)x0, cb, cb, shifts, 9, dW, 9 * cb, T, O, 1.f, 0.f, ws, wsb_conv,
                                     nullptr), NM_OK);
    // prune fused into the producer of g
    EXPECT(mvue_prune_2of4_producer(g, O, h, O, T, O, NM_BF16, 1, 2, 0, dense, O, vals, m16, nullptr), NM_OK);
    EXPECT(mvue_prune_1of2_producer(g, O, h, O, T, O, NM_F32, 1, 2, dense, O, vals, m16, nullptr), NM_OK);
    EXPECT(mvue_prune_2of4_producer(g, O, h, O, T, O, NM_BF16, 1, 2, 3, dense, O, vals, m16, nullptr), NM_ERR_UNSUPPORTED);
    EXPECT(mvue_prune_2of4_producer(g, O, nullptr, O, T, O, NM_BF16, 1, 2, 0, dense, O, vals, m16, nullptr), NM_ERR_NULL);
    EXPECT(mvue_prune_2of4_producer(g, O, h, O, T, O, NM_BF16, 1, 2, 0, g, O, vals, m16, nullptr), NM_ERR_ALIAS);
    EXPECT(mvue_prune_2of4_producer(g, O, h, O, T, O, NM_BF16, 1, 2, 0, dense, O, (char *)h + 64, m16, nullptr), NM_ERR_ALIAS);
    EXPECT(mvue_prune_2of4_producer(g, O, h, O - 8, T, O, NM_BF16, 1, 2, 0, dense, O, vals, m16, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4_producer(g, huge, h, huge, huge, O, NM_BF16, 1, 2, 0, dense, huge, vals, m16, nullptr), NM_ERR_SHAPE);
    // device-side scales of the 8-bit path
    alignas(16) static float rec_g[4], rec_h[4];
    EXPECT(nm_q8_scale(g, T, O, O, NM_BF16, 448.f, rec_g, nullptr), NM_OK);
    EXPECT(nm_q8_scale(g, T, O, O, NM_F32, 57344.f / 4.f, rec_h, nullptr), NM_OK);
    EXPECT(nm_cast_e4m3(h, T, I, I, NM_BF16, rec_h, (uint8_t *)x, I, nullptr), NM_OK);
    EXPECT(mvue_prune_2of4_q8_ds(g, T, O, O, NM_BF16, 1, 2, 0, rec_g, (uint8_t *)vals, m32, nullptr), NM_OK);
    EXPECT(mvue_prune_1of2_q8_ds(g, T, O, O, NM_BF16, 1, 2, rec_g, (uint8_t *)vals, m32, nullptr), NM_OK);
    EXPECT(mvue_prune_2of4_q8_t(g, T, O, T, NM_BF16, 1, 2, 0, -1.f, rec_g, (uint8_t *)vals, m32, nullptr), NM_OK);     // the record wins
    EXPECT(mvue_prune_1of2_q8_t(g, T, O, T, NM_BF16, 1, 2, 0.f, rec_g, (uint8_t *)vals, m32, nullptr), NM_OK);
    EXPECT(nm_update_gemm_q8_ds((const uint8_t *)vals, m32, (const uint8_t *)h, I, dW, I, T, O, I, rec_g, rec_h, 0.f, ws, wsb, nullptr), NM_OK);
    EXPECT(nm_update_gemm_q8_shifted_ds((const uint8_t *)vals, m32, (const uint8_t *)x0, cb, cb, shifts, 9, dW, 9 * cb, T, O, rec_g, rec_h, 0.f,
                                        ws, wsb_conv, nullptr), NM_OK);
    EXPECT(nm_q8_scale(g, T, O, O, NM_BF16, 0.f, rec_g, nullptr), NM_ERR_SHAPE);
    EXPECT(nm_q8_scale(g, T, O + 4, O + 4, NM_BF16, 1.f, rec_g, nullptr), NM_ERR_SHAPE);
    EXPECT(nm_q8_scale(g, T, O, O, NM_BF16, 1.f, nullptr, nullptr), NM_ERR_NULL);
    EXPECT(nm_q8_scale(g, T, O, O, NM_BF16, 1.f, (float *)((char *)g + 64), nullptr), NM_ERR_ALIAS);
    EXPECT(nm_q8_scale(g, huge, huge, huge, NM_BF16, 1.f, rec_g, nullptr), NM_ERR_SHAPE);
    EXPECT(nm_cast_e4m3(h, T, I + 8, I + 8, NM_BF16, rec_h, (uint8_t *)x, I + 8, nullptr), NM_ERR_SHAPE);
    EXPECT(nm_cast_e4m3(h, T, I, I, NM_BF16, rec_h, (uint8_t *)h + 32, I, nullptr), NM_ERR_ALIAS);
    EXPECT(nm_cast_e4m3(h, T, I, I, NM_BF16, nullptr, (uint8_t *)x, I, nullptr), NM_ERR_NULL);
    EXPECT(mvue_prune_2of4_q8_ds(g, T, O, O, NM_BF16, 1, 2, 0, nullptr, (uint8_t *)vals, m32, nullptr), NM_ERR_NULL);
    EXPECT(mvue_prune_2of4_q8_ds(g, T, O, O, NM_BF16, 1, 2, 0, rec_g + 1, (uint8_t *)vals, m32, nullptr), NM_ERR_ALIGN);
    EXPECT(nm_update_gemm_q8_ds((const uint8_t *)vals, m32, (const uint8_t *)h, I, dW, I, T, O, I, rec_g, nullptr, 0.f, ws, wsb, nullptr), NM_ERR_NULL);
    EXPECT(nm_update_gemm_q8_ds((const uint8_t *)vals, m32, (const uint8_t *)h, I, dW, I, T, O, I, dW + 4, rec_h, 0.f, ws, wsb, nullptr), NM_ERR_ALIAS);
    // the read/write-mix probe (pointers are never dereferenced on the host)
    EXPECT(nm_rw_mix_probe(g, (char *)g + (1ll << 40), 3, nullptr), NM_OK);
    EXPECT(nm_rw_mix_probe(g, (char *)g + 65536, 1, nullptr), NM_OK);
    EXPECT(nm_rw_mix_probe(g, (char *)g + 65536, 2, nullptr), NM_ERR_ALIAS);
    EXPECT(nm_rw_mix_probe(g, nullptr, 1, nullptr), NM_ERR_NULL);
    EXPECT(nm_rw_mix_probe((char *)g + 4, (char *)g + (1ll << 40), 1, nullptr), NM_ERR_ALIGN);
    EXPECT(nm_rw_mix_probe(g, g, -1, nullptr), NM_ERR_SHAPE);
    EXPECT(nm_rw_mix_probe(nullptr, nullptr, 0, nullptr), NM_OK);
    // empty problems do nothing and need no pointers
    EXPECT(mvue_prune_2of4(nullptr, 0, O, O, NM_BF16, 0, 0, 0, nullptr, nullptr, nullptr, 0, nullptr), NM_OK);
    EXPECT(mvue_prune_4of8_approx(nullptr, T, 0, 0, NM_BF16, 0, 0, nullptr, nullptr, nullptr, 0, nullptr), NM_OK);
    EXPECT(nm_update_gemm(nullptr, nullptr, nullptr, 0, dW, I, 0, O, I, NM_BF16, 0.f, nullptr, 0, nullptr), NM_OK);
    if (nm_update_gemm_workspace(T, O, I, NM_BF16) != wsb || nm_update_gemm_workspace(-1, O, I, NM_BF16) != 0) ++failures;

    // ---- rejecting paths: one of each kind per family of entry points
    EXPECT(mvue_prune_1of2(nullptr, T, O, O, NM_BF16, 0, 0, vals, m16, nullptr, 0, nullptr), NM_ERR_NULL);
    EXPECT(mvue_prune_2of4(g, T, O, O, NM_BF16, 0, 0, 0, nullptr, m16, nullptr, 0, nullptr), NM_ERR_NULL);
    EXPECT(mvue_prune_2of4(g, T + 4, O, O, NM_BF16, 0, 0, 0, vals, m16, nullptr, 0, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4(g, T, O + 4, O + 4, NM_BF16, 0, 0, 0, vals, m16, nullptr, 0, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4(g, T, O, O - 8, NM_BF16, 0, 0, 0, vals, m16, nullptr, 0, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4(g, -16, O, O, NM_BF16, 0, 0, 0, vals, m16, nullptr, 0, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4(g, T, O, O, 7, 0, 0, 0, vals, m16, nullptr, 0, nullptr), NM_ERR_DTYPE);
    EXPECT(mvue_prune_2of4(g, T, O, O, NM_BF16, 0, 0, 5, vals, m16, nullptr, 0, nullptr), NM_ERR_UNSUPPORTED);
    EXPECT(mvue_prune_2of4((char *)g + 2, T, O, O, NM_BF16, 0, 0, 0, vals, m16, nullptr, 0, nullptr), NM_ERR_ALIGN);
    EXPECT(mvue_prune_2of4(g, T, O, O + 4, NM_BF16, 0, 0, 0, vals, m16, nullptr, 0, nullptr), NM_ERR_ALIGN);
    EXPECT(mvue_prune_2of4(g, T, O, O, NM_BF16, 0, 0, 0, (char *)g + 64, m16, nullptr, 0, nullptr), NM_ERR_ALIAS);
    EXPECT(mvue_prune_2of4(g, T, O, O, NM_BF16, 0, 0, 0, vals, m16, (char *)vals + 16, O, nullptr), NM_ERR_ALIAS);
    EXPECT(mvue_prune_4of8_approx(g, T, O, O, NM_BF16, 0, 0, vals, (uint32_t *)((char *)vals + 32), nullptr, 0, nullptr), NM_ERR_ALIAS);
    EXPECT(mvue_prune_4of8_approx(g, T + 8, O, O, NM_BF16, 0, 0, vals, m32, nullptr, 0, nullptr), NM_ERR_SHAPE);
    EXPECT(nm_prune_greedy(g, T, O, O, NM_BF16, 4, 8, vals, m16, nullptr, 0, nullptr), NM_ERR_UNSUPPORTED);
    EXPECT(nm_compress(dense, T, O, O, NM_BF16, 3, 4, vals, m16, nullptr, nullptr), NM_ERR_UNSUPPORTED);
    EXPECT(mvue_prune_2of4_t(g, T, O, T - 16, NM_BF16, 0, 0, 0, vals, m16, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4_q8(g, T + 16, O, O, NM_BF16, 0, 0, 0, 1.f, (uint8_t *)vals, m32, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4_q8(g, T, O, O, NM_BF16, 0, 0, 0, -1.f, (uint8_t *)vals, m32, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4_q8_t(g, T, O, T, NM_BF16, 0, 0, 0, -1.f, nullptr, (uint8_t *)vals, m32, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4_q8_t(g, T, O, T - 32, NM_BF16, 0, 0, 0, 1.f, nullptr, (uint8_t *)vals, m32, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4_q8_t(g, T + 16, O, T + 16, NM_BF16, 0, 0, 0, 1.f, nullptr, (uint8_t *)vals, m32, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4_q8_t(g, T, O, T, NM_BF16, 0, 0, 2, 1.f, nullptr, (uint8_t *)vals, m32, nullptr), NM_ERR_UNSUPPORTED);
    EXPECT(mvue_prune_1of2_q8_t(g, T, O, T, NM_BF16, 0, 0, 1.f, nullptr, nullptr, m32, nullptr), NM_ERR_NULL);
    EXPECT(mvue_prune_1of2_q8_t(g, T, O, T, NM_BF16, 0, 0, 1.f, nullptr, (uint8_t *)g, m32, nullptr), NM_ERR_ALIAS);
    EXPECT(nm_update_gemm(vals, m16, h, I, dW, I, T, O, I, NM_BF16, 0.5f, ws, wsb, nullptr), NM_ERR_UNSUPPORTED);
    EXPECT(nm_update_gemm(vals, m16, h, I, dW, I, T, O, I, NM_BF16, 0.f, ws, wsb - 1, nullptr), NM_ERR_WORKSPACE);
    EXPECT(nm_update_gemm(vals, m16, h, I, dW, I, T, O, I, NM_BF16, 0.f, nullptr, 0, nullptr), NM_ERR_WORKSPACE);
    EXPECT(nm_update_gemm(vals, m16, h, I, dW, I, T, O, I, NM_BF16, 0.f, (char *)h + 256, wsb, nullptr), NM_ERR_ALIAS);
    EXPECT(nm_update_gemm(vals, m16, h, I, (float *)h, I, T, O, I, NM_BF16, 0.f, ws, wsb, nullptr), NM_ERR_ALIAS);
    EXPECT(nm_update_gemm(vals, m16, h, I - 8, dW, I, T, O, I, NM_BF16, 0.f, ws, wsb, nullptr), NM_ERR_SHAPE);
    EXPECT(nm_update_gemm(vals, m16, h, I, dW, I, T, O, I, 9, 0.f, ws, wsb, nullptr), NM_ERR_DTYPE);
    EXPECT(nm_update_gemm_q8((const uint8_t *)vals, m32, (const uint8_t *)h, I, dW, I, T, O, I, 1.f, 0.f, (char *)vals + 64, wsb, nullptr), NM_ERR_ALIAS);
    EXPECT(nm_update_gemm_shifted(vals, m16, x0, cb, cb, nullptr, 9, dW, 9 * cb, T, O, NM_BF16, 0.f, ws, wsb, nullptr), NM_ERR_NULL);
    EXPECT(nm_update_gemm_shifted(vals, m16, x0, cb, cb, shifts, 33, dW, 9 * cb, T, O, NM_BF16, 0.f, ws, wsb, nullptr), NM_ERR_SHAPE);
    EXPECT(nm_update_gemm_shifted(vals, m16, x0, cb, cb, shifts, 9, dW, 9 * cb, T, O, NM_BF16, 0.f, (char *)x0, wsb_conv, nullptr), NM_ERR_ALIAS);
    EXPECT(nm_update_gemm_q8_shifted((const uint8_t *)vals, m32, (const uint8_t *)x0, cb, cb, shifts, 9, dW, 9 * cb, T, O, 1.f, 0.f, (char *)dW,
                                     wsb_conv, nullptr), NM_ERR_ALIAS);
    // the static-scratch entry point: a problem whose split-K scratch exceeds the array
    EXPECT(nm_update_gemm_static(vals, m16, h, 4096, dW, 4096, T, 2048, 4096 / 16 * 2, NM_BF16, 0.f, nullptr), NM_OK);
    // absurd sizes: rejected as shapes, with no overflow in the range arithmetic on the way
    EXPECT(mvue_prune_2of4(g, huge, O, O, NM_BF16, 0, 0, 0, vals, m16, nullptr, 0, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4(g, T, huge, huge, NM_BF16, 0, 0, 0, vals, m16, nullptr, 0, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4(g, T, O, huge, NM_BF16, 0, 0, 0, vals, m16, nullptr, 0, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_4of8_approx(g, huge, huge, huge, NM_F32, 0, 0, vals, m32, dense, huge, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4_t(g, huge, O, huge, NM_BF16, 0, 0, 0, vals, m16, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4_q8(g, huge, huge, huge, NM_BF16, 0, 0, 0, 1.f, (uint8_t *)vals, m32, nullptr), NM_ERR_SHAPE);
    EXPECT(mvue_prune_2of4_q8_t(g, huge, huge, huge, NM_BF16, 0, 0, 0, 1.f, nullptr, (uint8_t *)vals, m32, nullptr), NM_ERR_SHAPE);
    EXPECT(nm_compress(dense, huge, huge, huge, NM_F32, 2, 4, vals, m16, nullptr, nullptr), NM_ERR_SHAPE);
    EXPECT(nm_update_gemm(vals, m16, h, I, dW, I, huge, O, I, NM_BF16, 0.f, ws, wsb, nullptr), NM_ERR_SHAPE);
    EXPECT(nm_update_gemm(vals, m16, h, I, dW, huge, T, O, I, NM_BF16, 0.f, ws, wsb, nullptr), NM_ERR_SHAPE);
    EXPECT(nm_update_gemm_q8((const uint8_t *)vals, m32, (const uint8_t *)h, I, dW, I, huge, huge, I, 1.f, 0.f, ws, wsb, nullptr), NM_ERR_SHAPE);
    EXPECT(nm_update_gemm_shifted(vals, m16, x0, cb, cb, shifts, 9, dW, 9 * cb, huge, O, NM_BF16, 0.f, ws, wsb, nullptr), NM_ERR_SHAPE);
    EXPECT(nm_update_gemm_q8_shifted((const uint8_t *)vals, m32, (const uint8_t *)x0, cb, cb, shifts, 9, dW, huge, T, O, 1.f, 0.f, ws, wsb, nullptr),
           NM_ERR_SHAPE);
    if (failures) { fprintf(stderr, "abi sanitizer driver: %d failures\n", failures); return 1; }
    printf("abi sanitizer driver ok (%d stub launches)\n", g_launches);
    return 0;
}
