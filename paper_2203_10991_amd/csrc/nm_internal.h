// Internal declarations shared by the translation units of libnm_mvue (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define NM_DT_F32 0
#define NM_DT_BF16 1
#define NM_DT_F32_BF16X3 2   // update GEMM only: binary32 operands, multiplied as three bf16 terms each

namespace nm {

// Output scale of the 8-bit update GEMM: a host value, or (inv_a != nullptr) value * inv_a[1] * inv_b[1] with the two
// factors read on the device -- element [1] of a scale record written by launch_q8_scale is the inverse scale; the
// GEMM launchers leave that product in inv_b[3] (the record's scratch slot) for their kernels.
struct AlphaArg {
    float value;
    const float *inv_a, *inv_b;
    AlphaArg(float v = 1.0f, const float *a = nullptr, const float *b = nullptr) : value(v), inv_a(a), inv_b(b) {}
};

hipError_t launch_prune(int dt, int m, int est, const void *g, int64_t T, int64_t O, int64_t ldg, uint64_t seed,
                        uint32_t stream_id, void *vals, uint16_t *meta, void *dense, int64_t ldd, hipStream_t st);

// prune fused into the producer of the neural gradient: g_l = u * d (eq. (2): d = f'(z_l), u = W^T g_{l+1}) is written
// dense to gout and pruned + compressed in the same pass
hipError_t launch_prune_producer(int dt, int m, int est, const void *u, int64_t ldu, const void *d, int64_t ldd, int64_t T, int64_t O,
                                 uint64_t seed, uint32_t stream_id, void *gout, int64_t ldgo, void *vals, uint16_t *meta, hipStream_t st);

// the same prunes for a gradient stored transposed: gT [O x T], row stride ldt (est 0 optimal 2:4, 1 approx-MVUE 2:4, 3 MVUE 1:2)
hipError_t launch_prune_transposed(int dt, int est, const void *gT, int64_t T, int64_t O, int64_t ldt, uint64_t seed,
                                   uint32_t stream_id, void *vals, uint16_t *meta, hipStream_t st);

// approx-MVUE 4:8 (four magnitude-proportional draws out of eight): vals [T/2 x O] in octet order, meta32 [T/16 x O]
hipError_t launch_prune_4of8_approx(int dt, const void *g, int64_t T, int64_t O, int64_t ldg, uint64_t seed, uint32_t stream_id,
                                    void *vals, uint32_t *meta32, void *dense, int64_t ldd, hipStream_t st);

hipError_t launch_compress(int dt, int m, const void *d, int64_t T, int64_t O, int64_t ld, void *vals,
                           uint16_t *meta, int32_t *bad, hipStream_t st);

// dW = beta*dW + decompress(vals, meta)^T h
hipError_t launch_update_gemm(int dt, const void *vals, const uint16_t *meta, const void *h, int64_t ldh,
                              float *dW, int64_t lddw, int64_t T, int64_t O, int64_t I, float beta,
                              void *workspace, size_t workspace_bytes, hipStream_t st);
size_t update_gemm_workspace(int dt, int64_t T, int64_t O, int64_t I);

// kernels behind launch_update_gemm: sparse MFMA for bf16, dense fp32 MFMA for binary32; both split the reduction
// axis into slabs for shapes with few output tiles and sum the partials with launch_splitk_reduce
hipError_t launch_update_gemm_smfmac(const void *vals, const uint16_t *meta, const void *h, int64_t ldh, float *dW,
                                     int64_t lddw, int64_t T, int64_t O, int64_t I, float beta, void *workspace,
                                     hipStream_t st);
size_t update_gemm_smfmac_workspace(int64_t T, int64_t O, int64_t I);
size_t update_gemm_smfmac_shifted_workspace(int64_t T, int64_t O, int64_t I);
// the same product with h given as n row-shifted views of one [rows x cb] matrix x (bf16): h[t][j*cb + c] = x[(t + rows[j])*ldx + c]
hipError_t launch_update_gemm_smfmac_shifted(const void *vals, const uint16_t *meta, const void *x, int64_t ldx, int64_t cb,
                                             const int64_t *rows, int n, float *dW, int64_t lddw, int64_t T, int64_t O,
                                             float beta, void *workspace, hipStream_t st);
hipError_t launch_update_gemm_f32(const void *vals, const uint16_t *meta, const void *h, int64_t ldh, float *dW,
                                  int64_t lddw, int64_t T, int64_t O, int64_t I, float beta, void *workspace,
                                  hipStream_t st);
size_t update_gemm_f32_workspace(int64_t T, int64_t O, int64_t I);

// binary32 operands split into three bf16 terms each, the six partial products as one run of the 16-bit sparse GEMM over
// operands stacked along the token axis (gemm_f32_split.hip)
hipError_t launch_update_gemm_f32_split(const void *vals, const uint16_t *meta, const void *h, int64_t ldh, float *dW,
                                        int64_t lddw, int64_t T, int64_t O, int64_t I, float beta, void *workspace,
                                        hipStream_t st);
size_t update_gemm_f32_split_workspace(int64_t T, int64_t O, int64_t I);
hipError_t launch_splitk_reduce(const float *part, int slabs, float *dW, int64_t lddw, int64_t O, int64_t I,
                                int accumulate, AlphaArg alpha, hipStream_t st);

// 8-bit path: 2:4 prune with e5m2 output (stochastic rounding) in 32-token groups, and its update GEMM
// dW = beta*dW + alpha * decompress(vals8, meta32)^T h8  (vals8 e5m2, h8 e4m3)
hipError_t launch_prune_q8(int dt, int est, const void *g, int64_t T, int64_t O, int64_t ldg, uint64_t seed,
                           uint32_t stream_id, float scale, const float *scale_dev, uint8_t *vals8, uint32_t *meta32, hipStream_t st);
// ... of a gradient stored transposed (gT [O x T], tokens contiguous)
hipError_t launch_prune_q8_transposed(int dt, int est, const void *gT, int64_t T, int64_t O, int64_t ldt, uint64_t seed,
                                      uint32_t stream_id, float scale, const float *scale_dev, uint8_t *vals8, uint32_t *meta32,
                                      hipStream_t st);
hipError_t launch_update_gemm_q8(const uint8_t *vals8, const uint32_t *meta32, const uint8_t *h8, int64_t ldh, float *dW,
                                 int64_t lddw, int64_t T, int64_t O, int64_t I, AlphaArg alpha, float beta, void *workspace,
                                 hipStream_t st);
size_t update_gemm_q8_workspace(int64_t T, int64_t O, int64_t I);
// ... with h8 given as n row-shifted views of one [rows x cb] matrix x8
hipError_t launch_update_gemm_q8_shifted(const uint8_t *vals8, const uint32_t *meta32, const uint8_t *x8, int64_t ldx, int64_t cb,
                                         const int64_t *rows, int n, float *dW, int64_t lddw, int64_t T, int64_t O,
                                         AlphaArg alpha, float beta, void *workspace, hipStream_t st);
size_t update_gemm_q8_shifted_workspace(int64_t T, int64_t O, int64_t I);

// 8-bit path, per-tensor scale and activation cast (q8_scale.hip).  rec: device float[4] = {s, 1/s, bits of max|t|, 0}
// with s the largest power of two such that s * max|t| <= top (1 for an all-zero or non-finite tensor).
hipError_t launch_q8_scale(int dt, const void *t, int64_t R, int64_t C, int64_t ld, float top, float *rec, hipStream_t st);
// h8 = e4m3(h * rec[0]), round to nearest even, magnitudes beyond 448 saturate
hipError_t launch_cast_e4m3(int dt, const void *h, int64_t R, int64_t C, int64_t ld, const float *rec, uint8_t *h8, int64_t ld8,
                            hipStream_t st);
// measurement aid: streams 64 KB in and 36 KB out per block (the 16-bit prune's read:write mix)
hipError_t launch_rw_mix_probe(const void *src, void *dst, int64_t n_blocks, hipStream_t st);

// The library's static device scratch array (nm_static.hip): its size, and its address on the current device
// (looked up once per device; no allocation).
size_t static_scratch_bytes();
hipError_t static_scratch(void **ptr);

}  // namespace nm
