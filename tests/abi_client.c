/*
 * A plain C program that uses the library the way a non-Python caller would: device memory from the HIP runtime,
 * the entry points of include/nm_mvue.h with raw pointers, nothing else.  One pass of the hot path (MVUE 2:4
 * prune + compress, then the update GEMM) on a small bf16 problem with ragged tiles, checked against the CPU
 * oracle (linked in: this is a test): compressed tensors bit for bit, dW within 1e-2 of the sum of absolute products.
 * Also walks the error paths that need no device.  Built by tests/build_abi_client.py; run by the GPU tests.
 * Exit status 0 = all checks passed.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "nm_mvue.h"

/* the oracle's C entry points used here (oracle/mvue_oracle.c) */
int oracle_prune_2of4(const void *g, int64_t T, int64_t O, int64_t ldg, int dt, uint64_t seed, uint32_t stream_id,
                      void *vals, uint16_t *meta, void *dense, int64_t ldd);
void oracle_update_gemm(const void *vals, const uint16_t *meta, const void *h, int64_t ldh, int64_t T, int64_t O,
                        int64_t I, int dt, double beta, const float *dW_in, double *dW, double *absdW);

#define HIP_OK(call)                                                                              \
    do {                                                                                          \
        hipError_t e_ = (call);                                                                   \
        if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_)); return 2; } \
    } while (0)
#define NM_OK_OR_FAIL(call)                                                                       \
    do {                                                                                          \
        int rc_ = (call);                                                                         \
        if (rc_ != 0) { fprintf(stderr, "%s -> %d: %s\n", #call, rc_, nm_last_error()); return 3; } \
    } while (0)

static uint64_t lcg_state = 0x2545F4914F6CDD1DULL;
static double uniform01(void)
{
    lcg_state = lcg_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (double)(lcg_state >> 11) / 9007199254740992.0;
}
/* heavy-tailed values with exact zeros, as bf16 bit patterns (truncated binary32) */
static uint16_t draw_bf16(double zero_share, double spread)
{
    if (uniform01() < zero_share) return 0;
    const float x = (float)((uniform01() - 0.5) * exp(spread * (uniform01() - 0.5)));
    uint32_t b;
    memcpy(&b, &x, 4);
    return (uint16_t)(b >> 16);
}

int main(void)
{
    const int64_t T = 16 * 21, O = 8 * 37, I = 16 * 9;     /* not multiples of any tile size */
    const uint64_t seed = 0x9E3779B97F4A7C15ULL;
    const uint32_t stream_id = 7;
    printf("%s; T=%lld O=%lld I=%lld\n", nm_version(), (long long)T, (long long)O, (long long)I);

    /* argument errors come back as codes with a message, before anything touches the device */
    if (mvue_prune_2of4(NULL, T, O, O, NM_BF16, seed, stream_id, 0, NULL, NULL, NULL, 0, NULL) == 0 || !nm_last_error()[0]) {
        fprintf(stderr, "NULL pointers were accepted\n");
        return 4;
    }
    if (mvue_prune_2of4((void *)0x1000, T + 1, O, O, NM_BF16, seed, stream_id, 0, (void *)0x100000, (uint16_t *)0x200000,
                        NULL, 0, NULL) == 0) {
        fprintf(stderr, "a token count that is no multiple of 16 was accepted\n");
        return 4;
    }

    uint16_t *g = malloc((size_t)(T * O) * 2), *h = malloc((size_t)(T * I) * 2);
    for (int64_t i = 0; i < T * O; ++i) g[i] = draw_bf16(0.3, 6.0);
    for (int64_t i = 0; i < T * I; ++i) h[i] = draw_bf16(0.0, 2.0);

    const size_t vals_bytes = (size_t)(T / 2 * O) * 2, meta_bytes = (size_t)(T / 16 * O) * 2, dw_bytes = (size_t)(O * I) * 4;
    void *d_g, *d_h, *d_vals, *d_meta, *d_dW, *d_ws = NULL;
    HIP_OK(hipSetDevice(0));
    HIP_OK(hipMalloc(&d_g, (size_t)(T * O) * 2));
    HIP_OK(hipMalloc(&d_h, (size_t)(T * I) * 2));
    HIP_OK(hipMalloc(&d_vals, vals_bytes));
    HIP_OK(hipMalloc(&d_meta, meta_bytes));
    HIP_OK(hipMalloc(&d_dW, dw_bytes));
    HIP_OK(hipMemcpy(d_g, g, (size_t)(T * O) * 2, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_h, h, (size_t)(T * I) * 2, hipMemcpyHostToDevice));
    const size_t ws_bytes = nm_update_gemm_workspace(T, O, I, NM_BF16);
    if (ws_bytes) HIP_OK(hipMalloc(&d_ws, ws_bytes));

    NM_OK_OR_FAIL(mvue_prune_2of4(d_g, T, O, O, NM_BF16, seed, stream_id, 0, d_vals, (uint16_t *)d_meta, NULL, 0, NULL));
    NM_OK_OR_FAIL(nm_update_gemm(d_vals, (const uint16_t *)d_meta, d_h, I, (float *)d_dW, I, T, O, I, NM_BF16, 0.0f,
                                 d_ws, ws_bytes, NULL));
    HIP_OK(hipDeviceSynchronize());

    uint16_t *vals = malloc(vals_bytes), *meta = malloc(meta_bytes);
    float *dW = malloc(dw_bytes);
    HIP_OK(hipMemcpy(vals, d_vals, vals_bytes, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(meta, d_meta, meta_bytes, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(dW, d_dW, dw_bytes, hipMemcpyDeviceToHost));

    uint16_t *o_vals = calloc(vals_bytes, 1), *o_meta = calloc(meta_bytes, 1);
    if (oracle_prune_2of4(g, T, O, O, NM_BF16, seed, stream_id, o_vals, o_meta, NULL, 0) != 0) return 5;
    if (memcmp(meta, o_meta, meta_bytes) != 0) { fprintf(stderr, "index metadata differs from the oracle\n"); return 6; }
    if (memcmp(vals, o_vals, vals_bytes) != 0) { fprintf(stderr, "kept values differ from the oracle\n"); return 6; }
    double *want = calloc((size_t)(O * I), 8), *wabs = calloc((size_t)(O * I), 8);
    oracle_update_gemm(o_vals, o_meta, h, I, T, O, I, NM_BF16, 0.0, NULL, want, wabs);
    double worst = 0.0;
    for (int64_t i = 0; i < O * I; ++i) {
        const double e = fabs((double)dW[i] - want[i]) / (wabs[i] > 1e-300 ? wabs[i] : 1e-300);
        if (!(e <= worst)) worst = e;                       /* (a NaN ends up in worst) */
    }
    printf("compressed tensors bit-exact; dW max |err| / sum|ab| = %.3e\n", worst);
    if (!(worst <= 1e-2)) { fprintf(stderr, "dW outside the tolerance\n"); return 7; }

    HIP_OK(hipFree(d_g)); HIP_OK(hipFree(d_h)); HIP_OK(hipFree(d_vals)); HIP_OK(hipFree(d_meta)); HIP_OK(hipFree(d_dW));
    if (d_ws) HIP_OK(hipFree(d_ws));
    free(g); free(h); free(vals); free(meta); free(dW); free(o_vals); free(o_meta); free(want); free(wabs);
    printf("abi client ok\n");
    return 0;
}
