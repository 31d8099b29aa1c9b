/*
 * nm_mvue.h -- C ABI of the MI355X (gfx950) library for minimum-variance unbiased N:M
 * pruning of neural gradients and the weight-update GEMM that consumes the pruned
 * operand (arXiv 2203.10991).
 *
 * Conventions
 *   g   [T x O]  neural gradient of a layer, row-major, row stride ldg (elements).  T = tokens
 *                (batch x positions, or N*H*W of a convolution written as im2col): the
 *                reduction axis of the update GEMM.  N:M blocks run ALONG T, so a block is M
 *                consecutive rows of one column.
 *   h   [T x I]  layer input (the other GEMM operand), row-major, row stride ldh.
 *   dW  [O x I]  binary32, row-major, row stride lddw:  dW = theta(g)^T h   (eq. (3)).
 *
 * Compressed operand ("group format"; the paper fixes none, it only counts the 2x footprint).
 * Tokens are cut into groups of 16 (= 4 quads = what one lane of a CDNA4 sparse-MFMA
 * instruction holds of the sparse operand).  For group G = t/16 and column o:
 *   vals[(G*O + o)*8 + 2*i + s]   s-th kept value (ascending position) of quad i (i = 0..3)
 *   meta[ G*O + o ]   (uint16)    bits [4i+1:4i]   = position (0..3) of kept value 0 of quad i
 *                                 bits [4i+3:4i+2] = position of kept value 1, kept0 < kept1
 * vals has T/2 * O elements of the tensor's dtype, meta T/16 * O uint16; both contiguous.
 * A 1:2-pruned tensor is stored in the same format (quad i = pairs 2i, 2i+1; kept0 in {0,1},
 * kept1 in {2,3}), i.e. as the 2:4 pattern it also is.
 *
 * All pointers are DEVICE pointers owned by the caller unless stated otherwise.  The library
 * allocates nothing, frees nothing and never synchronises: every call validates its
 * arguments on the host, enqueues its kernels on `hip_stream` (a hipStream_t; NULL = the
 * null stream) and returns.  Outputs must not overlap inputs.
 *
 * Errors: every entry point returns an nm_status (0 = ok).  Validation happens before any
 * device work: a validation error (codes 1-7) means nothing was enqueued and no output was
 * touched.  NM_ERR_LAUNCH means the HIP runtime refused one of the call's launches; a call may
 * consist of several kernels, earlier ones may already be queued, and the call's outputs (and
 * workspace) are then undefined.  nm_last_error() gives a thread-local message for the last
 * failing call on the calling thread.
 *
 * Shape rules (ragged sizes are rejected; zero-padding by the caller is exact because an
 * all-zero block stays zero):  T % 16 == 0, O % 8 == 0, I % 8 == 0 (GEMM), ldg/ldd/ldh/lddw
 * such that every row starts 16-byte aligned, base pointers 16-byte aligned.  T, O or I equal
 * to 0 is accepted and does nothing (dW is still scaled by beta).
 */
#ifndef NM_MVUE_H
#define NM_MVUE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    NM_OK = 0,
    NM_ERR_NULL = 1,        /* a required pointer is NULL */
    NM_ERR_SHAPE = 2,       /* negative / ragged size, leading dimension smaller than the row */
    NM_ERR_DTYPE = 3,       /* dtype is not an nm_dtype */
    NM_ERR_ALIGN = 4,       /* pointer or row stride not 16-byte aligned */
    NM_ERR_ALIAS = 5,       /* an output range overlaps an input range */
    NM_ERR_WORKSPACE = 6,   /* workspace missing or smaller than nm_update_gemm_workspace() */
    NM_ERR_UNSUPPORTED = 7, /* valid request this build does not implement */
    NM_ERR_LAUNCH = 8       /* the HIP runtime refused a launch (message has the HIP error); outputs undefined */
} nm_status;

/* NM_F32_BF16X3 is an arithmetic mode of nm_update_gemm for binary32 operands (see there); the prune and compress
 * entry points take NM_F32 or NM_BF16 only. */
typedef enum { NM_F32 = 0, NM_BF16 = 1, NM_F32_BF16X3 = 2 } nm_dtype;

/*
 * MVUE 1:2 prune + compress (Sec. 4.1, eq. (6); threshold sampling of App. B.1).
 * For every pair (a1, a2) = (g[2r][o], g[2r+1][o]) keeps a1 with probability
 * |a1|/(|a1|+|a2|) and emits sign(a_kept)*(|a1|+|a2|), rounded to nearest-even in `dtype`.
 * The uniform of pair row r, column o is Philox4x32-10 with key = seed, counter =
 * (blk/4 low, blk/4 high, stream_id, 0), word blk%4, top 24 bits, blk = r*O + o; the
 * result is a pure function of (g, T, O, dtype, seed, stream_id), whatever ldg or the launch.
 *   vals, meta   out, group format above.
 *   dense_out    out, optional (NULL = skip): theta(g) as a dense [T x O] tensor, stride ldd,
 *                pruned positions +0.
 */
int mvue_prune_1of2(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype,
                    uint64_t seed, uint32_t stream_id,
                    void *vals, uint16_t *meta, void *dense_out, int64_t ldd, void *hip_stream);

/*
 * MVUE 2:4 prune + compress.  mode 0 = the optimal estimator (Sec. 4.2 conditions, eqs. (12)
 * and (14); pair probabilities of App. A.2, cases 1-3), one uniform per quad, blk = (t/4)*O + o.
 * Kept values are a_i/p_i (eq. (8)): (a1+a2+a3+a4)/2 when no element dominates, otherwise the
 * dominant element unchanged and its partner a1+a2+a3; signs are those of the inputs.
 * mode 1 = approx-MVUE (Sec. 4.4): one element is drawn with probability a_i/sum, a second one
 * from the remaining three with probability a_j/(sum - a_i) (two uniforms per quad, a counter
 * stream of their own); both are kept with the value a_k/p_k, p_k the inclusion probability of
 * that section.  No ranking, six binary32 divisions per quad.  A zero is never drawn while a
 * non-zero remains; padding falls on the lowest-index zeros.
 * Any other mode returns NM_ERR_UNSUPPORTED.  Arguments as mvue_prune_1of2.
 * Non-finite values (every prune of this header): infinities and sums that overflow go through the same formulas in
 * IEEE arithmetic and the result is still a pure function of the arguments; a NaN makes the kept values of its block NaN,
 * and which positions of that block are kept is unspecified.
 */
int mvue_prune_2of4(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype,
                    uint64_t seed, uint32_t stream_id, int mode,
                    void *vals, uint16_t *meta, void *dense_out, int64_t ldd, void *hip_stream);

/*
 * mvue_prune_2of4 for a gradient that is stored transposed: gT is [O x T] with the tokens contiguous (row stride ldt
 * elements), as a producer that writes g^T leaves it; N:M blocks are then four adjacent elements of a row (the
 * "contiguous elements" of Sec. 1).  Same estimators (mode 0 / 1), random stream and block index as mvue_prune_2of4:
 * vals and meta equal what mvue_prune_2of4 writes for the transposed tensor, bit for bit.  No dense output.
 */
int mvue_prune_2of4_t(const void *gT, int64_t T, int64_t O, int64_t ldt, int dtype,
                      uint64_t seed, uint32_t stream_id, int mode, void *vals, uint16_t *meta, void *hip_stream);

/* The same for MVUE 1:2 (eq. (6)): equals mvue_prune_1of2 on the transposed tensor, bit for bit. */
int mvue_prune_1of2_t(const void *gT, int64_t T, int64_t O, int64_t ldt, int dtype,
                      uint64_t seed, uint32_t stream_id, void *vals, uint16_t *meta, void *hip_stream);

/*
 * MVUE 1:4 prune + compress (appendix, "Additional sparsity results": MVUE 1:2 on a block of four).
 * Of every quad one element survives: position k with probability |a_k|/sum|a|, emitting
 * sign(a_k)*sum|a| (eq. (6) with four terms; variance sum_k |a_k|(sum|a| - |a_k|)).  One uniform per quad,
 * the stream of mvue_prune_2of4 mode 0.  The output uses the 2:4 group format above -- gfx950's sparse
 * matrix instructions are 4:2 only -- with a +0 in the quad's second slot (at the lowest other position,
 * as nm_compress would pad), so nm_update_gemm consumes it unchanged.  Arguments as mvue_prune_1of2.
 */
int mvue_prune_1of4(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype,
                    uint64_t seed, uint32_t stream_id,
                    void *vals, uint16_t *meta, void *dense_out, int64_t ldd, void *hip_stream);

/*
 * MVUE prune fused into the PRODUCER of the neural gradient (eq. (2): g_l = Diag(f'(z_l)) W^T g_{l+1}; the dense
 * product u = W^T g_{l+1} is a GEMM the method leaves alone, the last step that makes g_l is the elementwise product
 * with the activation's derivative d = f'(z_l)).  One pass forms g_l = u * d (one binary32 product per element,
 * rounded to nearest even in `dtype`), writes it dense to g_out -- the next layer's backward GEMM reads it -- and
 * prunes + compresses it from registers, so g_l is never read back: 2 of the 3.125 bytes per element a separate
 * prune call moves (bf16) disappear.  vals and meta equal mvue_prune_2of4 / mvue_prune_1of2 of g_out for the same
 * (seed, stream_id, mode), bit for bit.
 *   u, d       [T x O] of `dtype`, row strides ldu, ldd     g_out  [T x O] of `dtype`, row stride ldg
 * (On this device the matrix pipeline idles while a GEMM epilogue selects -- ~90 vector instructions per quad -- so
 * the fusion point is this elementwise step and not the GEMM's own epilogue.)
 */
int mvue_prune_2of4_producer(const void *u, int64_t ldu, const void *d, int64_t ldd, int64_t T, int64_t O, int dtype,
                             uint64_t seed, uint32_t stream_id, int mode,
                             void *g_out, int64_t ldg, void *vals, uint16_t *meta, void *hip_stream);
int mvue_prune_1of2_producer(const void *u, int64_t ldu, const void *d, int64_t ldd, int64_t T, int64_t O, int dtype,
                             uint64_t seed, uint32_t stream_id,
                             void *g_out, int64_t ldg, void *vals, uint16_t *meta, void *hip_stream);

/*
 * approx-MVUE 4:8 prune + compress (appendix, "Additional sparsity results": the approximate 2:4 method of Sec. 4.4
 * carried over to more elements).  Of every block of eight consecutive tokens of a column four elements are drawn one
 * after the other without replacement, each with probability |a_j| / (sum of the magnitudes not yet drawn), and kept
 * with the value a_k / p_k (eq. (8)), p_k = the probability that k is among the four, computed exactly from its
 * definition (by the set of elements drawn so far; binary32, fixed operation order).  A block with at most four
 * non-zeros keeps them unchanged and pads with its lowest-index zeros; a zero is never drawn while a non-zero
 * remains.  Four uniforms per block: Philox4x32-10, key = seed, counter = (blk low, blk high, stream_id, 3),
 * blk = (t/8)*O + o, draw d uses the top 24 bits of word d.  Pure function of (g, T, O, dtype, seed, stream_id).
 * gfx950's sparse matrix instructions are 4:2 only, so the output is a storage format, not an operand of
 * nm_update_gemm (the appendix itself remarks that other ratios need other hardware):
 *     vals[(G*O + o)*8 + 4*b + s]   s-th kept value (ascending position) of octet b = 0, 1 of 16-token group G = t/16
 *     meta32[G*O + o]  (uint32)     bits [16b + 3s + 2 : 16b + 3s] = position (0..7) of that value inside the octet
 *     dense_out                     optional (NULL = skip): theta(g) as a dense [T x O] tensor, pruned positions +0
 * T % 16 == 0, O % 8 == 0; vals holds T/2 * O elements of the dtype, meta32 T/16 * O words.
 */
int mvue_prune_4of8_approx(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype,
                           uint64_t seed, uint32_t stream_id,
                           void *vals, uint32_t *meta32, void *dense_out, int64_t ldd, void *hip_stream);

/*
 * Greedy N:M prune + compress: the comparison method of the paper's tables (Sec. 4.1, 1:2 ablation table: the
 * traditional minimum-MSE method; Sec. 5: "keeping the N largest elements in each block").  (n,m) = (1,2) or (2,4):
 * of every block along T the n largest magnitudes are kept, values unchanged (bit for bit); among equal
 * magnitudes the lower position is kept.  Deterministic and BIASED: it exists to reproduce the paper's baseline,
 * not to train with.  Outputs as mvue_prune_1of2 (group format; optional dense_out).
 */
int nm_prune_greedy(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype, int n, int m,
                    void *vals, uint16_t *meta, void *dense_out, int64_t ldd, void *hip_stream);

/*
 * Deterministic compression of a dense [T x O] tensor that already is n:m sparse along T
 * ((n,m) = (1,2) or (2,4)) into the group format: the halved footprint the abstract counts.
 * Kept positions are the non-zero positions, padded with the lowest-index zero positions of
 * the block; values are copied bit for bit.  With the dense_out of a prune call as input it
 * reproduces that call's vals and meta exactly.
 *   bad_blocks   optional device int32 counter (NULL = do not count): incremented once per
 *                block that holds more than n non-zeros (such a block keeps its first n).
 *                The caller zeroes it and reads it after synchronising.
 */
int nm_compress(const void *dense, int64_t T, int64_t O, int64_t ld, int dtype, int n, int m,
                void *vals, uint16_t *meta, int32_t *bad_blocks, void *hip_stream);

/*
 * Update GEMM (eq. (3)):  dW[O x I] = beta*dW + decompress(vals, meta)^T h,  beta in {0, 1},
 * accumulation in binary32.  NM_BF16 runs on sparse MFMA (4:2 along the reduction axis) and
 * skips the pruned half of the products; NM_F32 has no sparse matrix instruction on gfx950
 * and expands the operand on the fly for dense fp32 MFMA (every product is executed).
 * NM_F32_BF16X3: the same binary32 tensors, but each value is split into three bf16 terms (24 significant bits)
 * and the six partial products of first and second order run on the sparse 16-bit path, accumulated in binary32:
 * |error| below 2^-22 of the sum of absolute products plus the accumulation's own rounding, at less than half the
 * time of NM_F32.  It needs a larger workspace: six bf16 copies of each operand live there, stacked along the token
 * axis so that one run of the 16-bit kernels sums the six products (6 x (T/2*O + T*I) x 2 bytes, plus the index
 * words six times).  A non-finite operand value makes the results it touches non-finite, but an infinity may come out
 * as a NaN.
 *   workspace    device scratch of at least nm_update_gemm_workspace(T,O,I,dtype) bytes
 *                (split-K partial sums); may be NULL when that size is 0.
 * O and ldh may not exceed 2^21 (NM_ERR_UNSUPPORTED): the kernels reach a few hundred rows of h
 * and a few dozen token groups of vals through 32-bit byte offsets.
 */
int nm_update_gemm(const void *vals, const uint16_t *meta, const void *h, int64_t ldh,
                   float *dW, int64_t lddw, int64_t T, int64_t O, int64_t I, int dtype, float beta,
                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Update GEMM of a convolution without the im2col matrix (App. B.1, part 1: activation A [B x C_I x H x W],
 * gradients G [B x C_O x H x W], update [C_I x C_O x k x k]).  The dense operand is given as n_shift row-shifted
 * views of ONE matrix x [rows x cb] (row stride ldx):
 *     h[t][j*cb + c] = x[(t + row_shift[j])*ldx + c],   j = 0..n_shift-1,   I = n_shift*cb,
 *     dW[O x I] = beta*dW + decompress(vals, meta)^T h.
 * For a k x k, stride-1 convolution: x is the zero-padded channels-last activation grid [N][H+2p][W+2p][C]
 * flattened to rows (cb = C), the gradient is pruned on the same padded grid (zeros on the border), and tap
 * (ky, kx) has row_shift = (ky-p)*(W+2p) + (kx-p); dW comes out as [O][ky][kx][C].
 *   x            device pointer to row 0.  Rows -m .. T+m-1, m = max|row_shift|, must be readable and hold finite
 *                values (zeros): border rows of the gradient, whose kept values are zero, are multiplied with them.
 *   row_shift    HOST array of n_shift (1..32) row shifts.
 * NM_BF16 only (NM_ERR_UNSUPPORTED otherwise); cb % 8 == 0; workspace of at least
 * nm_update_gemm_shifted_workspace(T, O, cb, n_shift) bytes (its own plan: not the size nm_update_gemm asks for).
 */
int nm_update_gemm_shifted(const void *vals, const uint16_t *meta, const void *x, int64_t ldx, int64_t cb,
                           const int64_t *row_shift, int n_shift, float *dW, int64_t lddw, int64_t T, int64_t O,
                           int dtype, float beta, void *workspace, size_t workspace_bytes, void *hip_stream);
size_t nm_update_gemm_shifted_workspace(int64_t T, int64_t O, int64_t cb, int n_shift);

/* Bytes of workspace nm_update_gemm needs for this problem (0 when it runs in one pass). */
size_t nm_update_gemm_workspace(int64_t T, int64_t O, int64_t I, int dtype);

/*
 * nm_update_gemm for callers that cannot allocate device memory or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks, kernels and results as
 * nm_update_gemm, without the workspace pair: the split-K partial sums go to a static device array inside the
 * library (nm_update_gemm_static_max() bytes, 64 MiB, held by every GPU the library runs on until the process
 * ends).  The call allocates and frees nothing.  A problem whose nm_update_gemm_workspace() exceeds that size
 * returns NM_ERR_WORKSPACE (nothing is enqueued); problems that need no workspace are unlimited.
 * All calls on one GPU share the array: two calls that may run at the same time on one GPU (different streams,
 * different threads) race on it.  Calls on one stream, or otherwise ordered, are safe; the array keeps the last
 * call's partial sums and every call overwrites what it reads.
 */
int nm_update_gemm_static(const void *vals, const uint16_t *meta, const void *h, int64_t ldh,
                          float *dW, int64_t lddw, int64_t T, int64_t O, int64_t I, int dtype, float beta,
                          void *hip_stream);
size_t nm_update_gemm_static_max(void);

/*
 * 8-bit neural gradients on top of 2:4 sparsity (Sec. 5: the rows that combine N:M sparsity in all
 * phases with 8-bit quantisation use FP8 neural gradients; Sec. 3: the quantiser of a neural gradient
 * has to be unbiased).  The paper fixes neither bit layout nor scale; this library takes OCP e5m2
 * for the gradients and OCP e4m3 for the activations (the pair gfx950's 8-bit sparse MFMA multiplies).
 *
 * mvue_prune_2of4_q8: selection and kept values exactly as mvue_prune_2of4 (same mode, same random
 * stream: the same seed gives the same mask), taken in binary32; each kept value is multiplied by
 * `scale` (> 0, finite; one binary32 product) and rounded stochastically to e5m2: with lo <= |x| < hi
 * neighbours on the e5m2 grid and f = (|x| - lo)/(hi - lo) the result is hi iff
 * r16 + floor(f * 2^16) >= 2^16, r16 uniform in [0, 2^16); |x| >= 57344 saturates to 57344, the
 * sign is kept; a NaN gives an e5m2 NaN (which of its codes is unspecified).  E[q]/scale = theta(g) up to 2^-16 of a grid step.  r16: Philox4x32-10, key = seed,
 * counter = (blk/4 low, blk/4 high, stream_id, 2), word blk%4; low half for the first kept value of
 * the quad, high half for the second; blk = (t/4)*O + o.
 * Output, the 8-bit group format (device pointers, 16-byte aligned): tokens in groups of 32 = 8 quads,
 *     vals8[(G*O + o)*16 + 2*i + s]   s-th kept value (ascending position) of quad i   (T/2 * O bytes)
 *     meta32[G*O + o]                 bits [4i+1:4i] = position of kept 0, [4i+3:4i+2] = kept 1
 * T must be a multiple of 32, O of 8.  g: NM_F32 or NM_BF16, row stride ldg.
 */
int mvue_prune_2of4_q8(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype,
                       uint64_t seed, uint32_t stream_id, int mode, float scale,
                       uint8_t *vals8, uint32_t *meta32, void *hip_stream);

/*
 * The same for MVUE 1:2 (eq. (6)): quad i of a group holds the pairs 2i and 2i+1, the kept value of the first is
 * slot 2i (position 0 or 1), that of the second slot 2i+1 (position 2 or 3).  Selection as in mvue_prune_1of2 (same
 * stream, block index = pair row * O + o); the value, times scale, is rounded with the LOW half of the pair block's
 * rounding word (same counter layout as above, last counter word 2).  Consumed by nm_update_gemm_q8.
 */
int mvue_prune_1of2_q8(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype,
                       uint64_t seed, uint32_t stream_id, float scale,
                       uint8_t *vals8, uint32_t *meta32, void *hip_stream);

/*
 * The 8-bit prunes for a gradient stored transposed (gT [O x T], tokens contiguous, row stride ldt elements; see
 * mvue_prune_2of4_t): same selection, scaling, rounding, random streams and block indices, so vals8 and meta32 equal
 * what mvue_prune_2of4_q8 / mvue_prune_1of2_q8 write for the transposed tensor, bit for bit.  The scale: scale_rec
 * (device, a record of nm_q8_scale, 16-byte aligned) when it is not NULL -- the kept values are multiplied by
 * scale_rec[0] and `scale` is ignored --, else the host value `scale` (> 0, finite).  T a multiple of 32, O of 8.
 */
int mvue_prune_2of4_q8_t(const void *gT, int64_t T, int64_t O, int64_t ldt, int dtype,
                         uint64_t seed, uint32_t stream_id, int mode, float scale, const float *scale_rec,
                         uint8_t *vals8, uint32_t *meta32, void *hip_stream);
int mvue_prune_1of2_q8_t(const void *gT, int64_t T, int64_t O, int64_t ldt, int dtype,
                         uint64_t seed, uint32_t stream_id, float scale, const float *scale_rec,
                         uint8_t *vals8, uint32_t *meta32, void *hip_stream);

/*
 * Update GEMM (eq. (3)) on the 8-bit operands:
 *     dW[O x I] = beta*dW + alpha * decompress(vals8, meta32)^T h8,   beta in {0, 1},
 * h8 [T x I] e4m3 with row stride ldh (bytes = elements), products exact and accumulation in binary32
 * on the 8-bit sparse MFMA; alpha undoes the scales of the two operands.  I must be a multiple of 16,
 * ldh a multiple of 16; limits and workspace as nm_update_gemm (size from nm_update_gemm_q8_workspace).
 */
int nm_update_gemm_q8(const uint8_t *vals8, const uint32_t *meta32, const uint8_t *h8, int64_t ldh,
                      float *dW, int64_t lddw, int64_t T, int64_t O, int64_t I, float alpha, float beta,
                      void *workspace, size_t workspace_bytes, void *hip_stream);
size_t nm_update_gemm_q8_workspace(int64_t T, int64_t O, int64_t I);

/*
 * Measurement aid (no passage of the paper: a benchmark's yardstick).  Streams n_blocks * 64 KiB from src and writes
 * n_blocks * 36 KiB to dst with fully contiguous 4 KiB instructions -- the 16:9 read:write mix of the 16-bit
 * prune + compress (Sec. 4: the gradient in, half the values and 1/16 index words out) -- so that the prune kernel's
 * rate can be stated against what this mix reaches on the device.  With src and dst as arrays of 16-byte words,
 * block b and t = 0..255:  dst[(9b + k)*256 + t] = src[(16b + k)*256 + t] XOR src[(16b + k + 7)*256 + t], k = 0..8.
 * src, dst: device pointers, 16-byte aligned, not overlapping; the caller owns both.  Errors as everywhere.
 */
int nm_rw_mix_probe(const void *src, void *dst, int64_t n_blocks, void *hip_stream);

/*
 * Per-tensor scales of the 8-bit path without a host round trip (Sec. 5, 8-bit rows; the paper fixes no scale rule:
 * this library uses one power-of-two scale per tensor from its current maximum magnitude).
 *
 * nm_q8_scale writes a SCALE RECORD, four floats in device memory (16-byte aligned):
 *     rec[0] = s    the largest power of two with s * max|t| <= top, exponent kept in [-126, 126];
 *                   1 for an all-zero tensor or a maximum that is not finite
 *     rec[1] = 1/s  rec[2] = the bit pattern of max|t|   rec[3] = 0 (scratch of the record's consumer, see below)
 * t: [R x C] of NM_F32 or NM_BF16, row stride ld, C % 8 == 0.  top: the largest magnitude the 8-bit format is to
 * hold: 448 for e4m3 activations; 57344/4 for e5m2 gradients pruned 2:4 and 57344/2 for 1:2 (a kept value is at most
 * the sum of its block's magnitudes).  Three small kernels on the stream; the maximum is an order-independent atomic,
 * so the record is reproducible.
 *
 * nm_cast_e4m3: h8[r][c] = e4m3(h[r][c] * rec[0]) -- one binary32 product, round to nearest even, magnitudes beyond
 * 448 saturate to 448 -- for the activations of nm_update_gemm_q8.  C % 16 == 0, ld8 % 16 == 0 (bytes).
 *
 * The _ds ("device scale") forms of the 8-bit entry points read their scales from such records instead of host
 * arguments: mvue_prune_*_q8_ds multiplies kept values by rec[0]; nm_update_gemm_q8*_ds uses
 * alpha = rec_g[1] * rec_h[1], which a one-thread kernel of the call leaves in rec_h[3] for its GEMM kernels (so two
 * GEMM calls that may run at the same time must not share an activation record).  Everything else as the
 * host-scale forms.
 */
int nm_q8_scale(const void *t, int64_t R, int64_t C, int64_t ld, int dtype, float top, float *scale_rec, void *hip_stream);
int nm_cast_e4m3(const void *h, int64_t R, int64_t C, int64_t ld, int dtype, const float *scale_rec,
                 uint8_t *h8, int64_t ld8, void *hip_stream);
int mvue_prune_2of4_q8_ds(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype,
                          uint64_t seed, uint32_t stream_id, int mode, const float *scale_rec,
                          uint8_t *vals8, uint32_t *meta32, void *hip_stream);
int mvue_prune_1of2_q8_ds(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype,
                          uint64_t seed, uint32_t stream_id, const float *scale_rec,
                          uint8_t *vals8, uint32_t *meta32, void *hip_stream);
int nm_update_gemm_q8_ds(const uint8_t *vals8, const uint32_t *meta32, const uint8_t *h8, int64_t ldh,
                         float *dW, int64_t lddw, int64_t T, int64_t O, int64_t I,
                         const float *scale_rec_g, float *scale_rec_h, float beta,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The 8-bit update GEMM with the dense operand as row-shifted views (nm_update_gemm_shifted for the operands of
 * nm_update_gemm_q8: the paper's 8-bit rows are convolutional networks):
 *     dW[O x n_shift*cb] = beta*dW + alpha * decompress(vals8, meta32)^T h8,   h8[t][j*cb + c] = x8[(t + row_shift[j])*ldx + c].
 * x8: e4m3 codes; rows -m .. T+m-1 (m = max|row_shift|) readable and finite (zero codes).  cb % 16 == 0, T % 32 == 0.
 */
int nm_update_gemm_q8_shifted(const uint8_t *vals8, const uint32_t *meta32, const uint8_t *x8, int64_t ldx, int64_t cb,
                              const int64_t *row_shift, int n_shift, float *dW, int64_t lddw, int64_t T, int64_t O,
                              float alpha, float beta, void *workspace, size_t workspace_bytes, void *hip_stream);
size_t nm_update_gemm_q8_shifted_workspace(int64_t T, int64_t O, int64_t cb, int n_shift);
/* ... with alpha = scale_rec_g[1] * scale_rec_x[1] read on the device (see nm_q8_scale) */
int nm_update_gemm_q8_shifted_ds(const uint8_t *vals8, const uint32_t *meta32, const uint8_t *x8, int64_t ldx, int64_t cb,
                                 const int64_t *row_shift, int n_shift, float *dW, int64_t lddw, int64_t T, int64_t O,
                                 const float *scale_rec_g, float *scale_rec_x, float beta,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

/* Message of the last error on this thread ("" if none).  Static storage; do not free. */
const char *nm_last_error(void);

/* Build identification, e.g. "nm_mvue 0.1 gfx950". */
const char *nm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* NM_MVUE_H */
