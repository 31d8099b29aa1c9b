/*
 * Sanitizer driver for the CPU oracle (test infrastructure): built together with oracle/mvue_oracle.c under
 * -fsanitize=address,undefined and run by tests/test_sanitizers.py.  It walks every tensor-level entry point on
 * exactly-sized heap buffers (so that any access past an end is caught), with ragged shapes (column counts that are
 * not a multiple of anything but 8, padded row strides) and edge values (zeros, signed zeros, ties, subnormals, the
 * largest finite values), and the block-level functions on the same edge values.  Exit status 0 = no report.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
void oracle_select_1of2(const float x[2], float eps, int *kept, float *value);
void oracle_select_2of4(const float x[4], float eps, int pos[2], float value[2], int *which_case);
void oracle_select_2of4_approx(const float x[4], float eps1, float eps2, int pos[2], float value[2]);
void oracle_select_1of4(const float x[4], float eps, int *kept, float *value);
void oracle_select_greedy(const float *x, int m, int n, int *pos);
void oracle_select_4of8_approx(const float x[8], const float eps[4], int pos[4], float value[4]);
int oracle_prune_1of2(const void *, int64_t, int64_t, int64_t, int, uint64_t, uint32_t, void *, uint16_t *, void *, int64_t);
int oracle_prune_2of4(const void *, int64_t, int64_t, int64_t, int, uint64_t, uint32_t, void *, uint16_t *, void *, int64_t);
int oracle_prune_2of4_approx(const void *, int64_t, int64_t, int64_t, int, uint64_t, uint32_t, void *, uint16_t *, void *, int64_t);
int oracle_prune_1of4(const void *, int64_t, int64_t, int64_t, int, uint64_t, uint32_t, void *, uint16_t *, void *, int64_t);
int oracle_prune_greedy(const void *, int64_t, int64_t, int64_t, int, int, int, void *, uint16_t *, void *, int64_t);
int oracle_prune_4of8_approx(const void *, int64_t, int64_t, int64_t, int, uint64_t, uint32_t, void *, uint32_t *, void *, int64_t);
int64_t oracle_nm_compress(const void *, int64_t, int64_t, int64_t, int, int, int, void *, uint16_t *);
void oracle_nm_decompress(const void *, const uint16_t *, int64_t, int64_t, int, void *, int64_t);
void oracle_nm_decompress_4of8(const void *, const uint32_t *, int64_t, int64_t, int, void *, int64_t);
void oracle_update_gemm(const void *, const uint16_t *, const void *, int64_t, int64_t, int64_t, int64_t, int, double,
                        const float *, double *, double *);
void oracle_update_gemm_entries(const void *, const uint16_t *, const void *, int64_t, int64_t, int64_t, int64_t, int,
                                const int64_t *, int64_t, double *, double *);
uint8_t oracle_sr_e5m2(float x, uint32_t r16);
double oracle_e5m2_value(uint8_t c);
double oracle_e4m3_value(uint8_t c);
int oracle_prune_2of4_q8(const void *, int64_t, int64_t, int64_t, int, uint64_t, uint32_t, int, float, uint8_t *, uint32_t *);
int oracle_prune_1of2_q8(const void *, int64_t, int64_t, int64_t, int, uint64_t, uint32_t, float, uint8_t *, uint32_t *);
void oracle_update_gemm_q8(const uint8_t *, const uint32_t *, const uint8_t *, int64_t, int64_t, int64_t, int64_t, double,
                           const int64_t *, int64_t, double *, double *);
void oracle_update_gemm_shifted(const void *, const uint16_t *, const void *, int64_t, int64_t, const int64_t *, int, int64_t,
                                int64_t, int, double *, double *);
void oracle_update_gemm_q8_shifted(const uint8_t *, const uint32_t *, const uint8_t *, int64_t, int64_t, const int64_t *, int,
                                   int64_t, int64_t, double, double *, double *);

static const float EDGE[] = { 0.0f, -0.0f, 1.0f, -1.0f, 1.0f, 3.0f, -3.0f, 1e-45f, -1e-40f, 1e-38f, 3.0e38f, -3.0e38f,
                              1e30f, 1e-30f, 0.5f, 65504.0f, 7.0f, 7.0f, -7.0f, 2.5f };
#define N_EDGE ((int)(sizeof EDGE / sizeof EDGE[0]))

static uint64_t state = 88172645463325252ULL;
static uint32_t rnd(void) { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return (uint32_t)(state >> 16); }
static float draw(void)
{
    uint32_t r = rnd();
    if (r % 4 == 0) return 0.0f;
    if (r % 7 == 0) return EDGE[rnd() % N_EDGE] * 1e-3f;           /* scaled so that sums of eight stay finite */
    return ((r & 1) ? 1.0f : -1.0f) * expf(((float)(rnd() % 2000) - 1000.0f) / 200.0f);
}
static uint16_t to_bf16(float f) { uint32_t b; memcpy(&b, &f, 4); return (uint16_t)(b >> 16); }

static void *xmalloc(size_t n) { void *p = malloc(n ? n : 1); if (!p) { fprintf(stderr, "out of memory\n"); exit(2); } return p; }

static int run_tensor_case(int dt, int64_t T, int64_t O, int64_t I, int64_t ldg, int64_t ldh)
{
    const size_t es = dt == 0 ? 4 : 2;
    /* exactly sized: the last row holds O (I) elements only */
    void *g = xmalloc(((size_t)(T - 1) * ldg + O) * es), *h = xmalloc(((size_t)(T - 1) * ldh + I) * es);
    for (int64_t t = 0; t < T; ++t)
        for (int64_t o = 0; o < O; ++o) {
            float v = draw();
            if (dt == 0) ((float *)g)[t * ldg + o] = v; else ((uint16_t *)g)[t * ldg + o] = to_bf16(v);
        }
    for (int64_t t = 0; t < T; ++t)
        for (int64_t i = 0; i < I; ++i) {
            float v = draw();
            if (dt == 0) ((float *)h)[t * ldh + i] = v; else ((uint16_t *)h)[t * ldh + i] = to_bf16(v);
        }
    void *vals = xmalloc((size_t)(T / 2) * O * es), *dense = xmalloc(((size_t)(T - 1) * (O + 8) + O) * es);
    uint16_t *meta = xmalloc((size_t)(T / 16) * O * 2);
    uint32_t *meta32 = xmalloc((size_t)(T / 16) * O * 4);
    void *back = xmalloc((size_t)T * O * es);
    double *dW = xmalloc((size_t)O * I * 8), *aW = xmalloc((size_t)O * I * 8);
    int bad = 0;
    typedef int (*prune_fn)(const void *, int64_t, int64_t, int64_t, int, uint64_t, uint32_t, void *, uint16_t *, void *, int64_t);
    prune_fn fns[4] = { oracle_prune_1of2, oracle_prune_2of4, oracle_prune_2of4_approx, oracle_prune_1of4 };
    for (int f = 0; f < 4; ++f) {
        bad |= fns[f](g, T, O, ldg, dt, 0x123456789ULL + f, 5, vals, meta, dense, O + 8) != 0;
        bad |= fns[f](g, T, O, ldg, dt, 7, 0, vals, meta, NULL, 0) != 0;
        oracle_nm_decompress(vals, meta, T, O, dt, back, O);
        oracle_update_gemm(vals, meta, h, ldh, T, O, I, dt, 0.0, NULL, dW, aW);
        oracle_update_gemm(vals, meta, h, ldh, T, O, I, dt, 0.0, NULL, dW, NULL);
    }
    for (int n = 1; n <= 2; ++n) {
        bad |= oracle_prune_greedy(g, T, O, ldg, dt, n, 2 * n, vals, meta, dense, O + 8) != 0;
        bad |= oracle_nm_compress(dense, T, O, O + 8, dt, n, 2 * n, vals, meta) != 0;
    }
    bad |= oracle_prune_4of8_approx(g, T, O, ldg, dt, 99, 1, vals, meta32, dense, O + 8) != 0;
    oracle_nm_decompress_4of8(vals, meta32, T, O, dt, back, O);
    bad |= oracle_prune_2of4(g, T, O, ldg, dt, 1, 1, vals, meta, NULL, 0) != 0;
    int64_t oi[6] = { 0, 0, O - 1, I - 1, O / 2, I / 2 };
    double e[3], ea[3];
    oracle_update_gemm_entries(vals, meta, h, ldh, T, O, I, dt, oi, 3, e, ea);
    if (dt == 1 && T % 32 == 0) {
        uint8_t *v8 = xmalloc((size_t)(T / 2) * O), *h8 = xmalloc((size_t)(T - 1) * ldh + I);
        uint32_t *m32 = xmalloc((size_t)(T / 32) * O * 4);
        for (int64_t t = 0; t < T; ++t) for (int64_t i = 0; i < I; ++i) h8[t * ldh + i] = (uint8_t)(rnd() % 0x7e);
        for (int mode = 0; mode < 2; ++mode) bad |= oracle_prune_2of4_q8(g, T, O, ldg, dt, 3, 2, mode, 0.125f, v8, m32) != 0;
        oracle_update_gemm_q8(v8, m32, h8, ldh, T, O, I, 0.5, NULL, 0, dW, aW);
        oracle_update_gemm_q8(v8, m32, h8, ldh, T, O, I, 0.5, oi, 3, e, ea);
        bad |= oracle_prune_1of2_q8(g, T, O, ldg, dt, 3, 2, 4.0f, v8, m32) != 0;
        free(v8); free(h8); free(m32);
    }
    free(g); free(h); free(vals); free(dense); free(meta); free(meta32); free(back); free(dW); free(aW);
    return bad;
}

static int run_shifted_case(void)
{
    /* a 3x3 convolution's update GEMM on row-shifted views: x with exactly `margin` rows before and after */
    const int64_t T = 64, O = 16, C = 8, Wp = 6, margin = Wp + 1;
    uint16_t *g = xmalloc((size_t)T * O * 2), *xf = xmalloc((size_t)(T + 2 * margin) * C * 2);
    for (int64_t k = 0; k < T * O; ++k) g[k] = to_bf16(draw());
    for (int64_t k = 0; k < (T + 2 * margin) * C; ++k) xf[k] = to_bf16(draw());
    uint16_t *vals = xmalloc((size_t)(T / 2) * O * 2), *meta = xmalloc((size_t)(T / 16) * O * 2);
    int bad = oracle_prune_2of4(g, T, O, O, 1, 11, 0, vals, meta, NULL, 0) != 0;
    int64_t sh[9];
    for (int ky = 0; ky < 3; ++ky) for (int kx = 0; kx < 3; ++kx) sh[3 * ky + kx] = (ky - 1) * Wp + (kx - 1);
    double *dW = xmalloc((size_t)O * 9 * C * 8), *aW = xmalloc((size_t)O * 9 * C * 8);
    oracle_update_gemm_shifted(vals, meta, xf + margin * C, C, C, sh, 9, T, O, 1, dW, aW);
    uint8_t *v8 = xmalloc((size_t)(T / 2) * O), *x8 = xmalloc((size_t)(T + 2 * margin) * C);
    uint32_t *m32 = xmalloc((size_t)(T / 32) * O * 4);
    for (int64_t k = 0; k < (T + 2 * margin) * C; ++k) x8[k] = (uint8_t)(rnd() % 0x7e);
    bad |= oracle_prune_2of4_q8(g, T, O, O, 1, 11, 0, 0, 1.0f, v8, m32) != 0;
    oracle_update_gemm_q8_shifted(v8, m32, x8 + margin * C, C, C, sh, 9, T, O, 1.0, dW, aW);
    free(g); free(xf); free(vals); free(meta); free(dW); free(aW); free(v8); free(x8); free(m32);
    return bad;
}

int main(void)
{
    int bad = 0;
    /* block-level functions on every combination of edge values that fits, at the extreme uniforms */
    const float eps_list[3] = { 0.0f, 0.5f, 1.0f - 0x1p-24f };
    for (int a = 0; a < N_EDGE; ++a)
        for (int b = 0; b < N_EDGE; ++b)
            for (int e = 0; e < 3; ++e) {
                float x2[2] = { EDGE[a], EDGE[b] };
                int k; float v;
                oracle_select_1of2(x2, eps_list[e], &k, &v);
                bad |= k < 0 || k > 1;
                float x4[4] = { EDGE[a], EDGE[b], EDGE[(a + b) % N_EDGE], EDGE[(a * 3 + b) % N_EDGE] };
                int pos[4], wc; float val[4];
                oracle_select_2of4(x4, eps_list[e], pos, val, &wc);
                bad |= pos[0] < 0 || pos[0] >= pos[1] || pos[1] > 3;
                oracle_select_2of4_approx(x4, eps_list[e], eps_list[(e + 1) % 3], pos, val);
                bad |= pos[0] < 0 || pos[0] >= pos[1] || pos[1] > 3;
                oracle_select_1of4(x4, eps_list[e], &k, &v);
                bad |= k < 0 || k > 3;
                oracle_select_greedy(x4, 4, 2, pos);
                bad |= pos[0] < 0 || pos[0] >= pos[1] || pos[1] > 3;
                float x8[8], ee[4] = { eps_list[e], eps_list[(e + 1) % 3], eps_list[(e + 2) % 3], eps_list[e] };
                for (int j = 0; j < 8; ++j) x8[j] = EDGE[(a + j * b + j) % N_EDGE] * 0.1f;
                oracle_select_4of8_approx(x8, ee, pos, val);
                for (int s = 0; s < 4; ++s) bad |= pos[s] < 0 || pos[s] > 7 || (s && pos[s] <= pos[s - 1]);
            }
    for (int c = 0; c < 256; ++c) { (void)oracle_e5m2_value((uint8_t)c); (void)oracle_e4m3_value((uint8_t)c); }
    for (int a = 0; a < N_EDGE; ++a) for (uint32_t r = 0; r < 65536; r += 4369) (void)oracle_sr_e5m2(EDGE[a], r);
    /* tensors: ragged column counts, padded strides, both dtypes */
    bad |= run_tensor_case(0, 16, 8, 8, 8, 8);
    bad |= run_tensor_case(0, 48, 24, 40, 33, 47);
    bad |= run_tensor_case(1, 32, 8, 16, 8, 16);
    bad |= run_tensor_case(1, 96, 40, 48, 56, 64);
    bad |= run_tensor_case(1, 64, 72, 16, 72, 16);
    bad |= run_shifted_case();
    if (bad) { fprintf(stderr, "oracle sanitizer driver: a call returned an error or an index out of range\n"); return 1; }
    printf("oracle sanitizer driver ok\n");
    return 0;
}
