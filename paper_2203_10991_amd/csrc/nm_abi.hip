// C ABI of libnm_mvue: host-side argument validation and kernel dispatch.
// Every check runs before any device work; no allocation, no synchronisation.
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/nm_mvue.h"
#include "nm_internal.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

inline int64_t esize(int dt) { return dt == NM_BF16 ? 2 : 4; }
inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

struct Range { uintptr_t lo, hi; const char *name; };
inline Range range_of(const void *p, int64_t bytes, const char *name)
{
    return Range{(uintptr_t)p, (uintptr_t)p + (bytes > 0 ? (uintptr_t)bytes : 0), name};
}
// rows x stride elements must stay far below 2^63 bytes: every byte range below is formed without overflow
inline bool too_big(int64_t rows, int64_t stride)
{
    const int64_t lim = (int64_t)1 << 58;
    return rows > lim || stride > lim || (rows > 0 && stride > 0 && rows > lim / stride);
}
inline bool overlap(const Range &a, const Range &b) { return a.lo < b.hi && b.lo < a.hi && a.lo != a.hi && b.lo != b.hi; }

// shape / dtype / pointer checks shared by the two prune calls and nm_compress
int check_tensor(const char *fn, const void *g, int64_t T, int64_t O, int64_t ld, int dt, const char *what)
{
    if (dt != NM_F32 && dt != NM_BF16) return fail(NM_ERR_DTYPE, "%s: dtype %d is not NM_F32 (0) or NM_BF16 (1)", fn, dt);
    if (T < 0 || O < 0) return fail(NM_ERR_SHAPE, "%s: negative size T=%lld O=%lld", fn, (long long)T, (long long)O);
    if (T % 16) return fail(NM_ERR_SHAPE, "%s: T=%lld is not a multiple of 16 (pad with zero rows)", fn, (long long)T);
    if (O % 8) return fail(NM_ERR_SHAPE, "%s: O=%lld is not a multiple of 8 (pad with zero columns)", fn, (long long)O);
    if (too_big(T, O) || too_big(T, ld)) return fail(NM_ERR_SHAPE, "%s: %s is larger than 2^58 elements", fn, what);
    if (T == 0 || O == 0) return NM_OK;
    if (!g) return fail(NM_ERR_NULL, "%s: %s is NULL", fn, what);
    if (ld < O) return fail(NM_ERR_SHAPE, "%s: row stride %lld of %s is smaller than O=%lld", fn, (long long)ld, what, (long long)O);
    if (!aligned16(g) || (ld * esize(dt)) % 16)
        return fail(NM_ERR_ALIGN, "%s: %s needs a 16-byte aligned base and row stride", fn, what);
    return NM_OK;
}

int check_outputs(const char *fn, const void *in, int64_t T, int64_t O, int64_t ld, int dt, const void *vals,
                  const void *meta, const void *dense, int64_t ldd)
{
    if (T == 0 || O == 0) return NM_OK;
    if (!vals) return fail(NM_ERR_NULL, "%s: vals is NULL", fn);
    if (!meta) return fail(NM_ERR_NULL, "%s: meta is NULL", fn);
    if (!aligned16(vals) || !aligned16(meta)) return fail(NM_ERR_ALIGN, "%s: vals and meta need 16-byte aligned bases", fn);
    const int64_t es = esize(dt);
    Range rin = range_of(in, ((T - 1) * ld + O) * es, "input");
    Range rv = range_of(vals, T / 2 * O * es, "vals");
    Range rm = range_of(meta, T / 16 * O * 2, "meta");
    if (overlap(rin, rv) || overlap(rin, rm) || overlap(rv, rm))
        return fail(NM_ERR_ALIAS, "%s: input, vals and meta must not overlap", fn);
    if (dense) {
        if (ldd < O || too_big(T, ldd)) return fail(NM_ERR_SHAPE, "%s: ldd=%lld is smaller than O=%lld (or beyond 2^58 elements)", fn, (long long)ldd, (long long)O);
        if (!aligned16(dense) || (ldd * es) % 16) return fail(NM_ERR_ALIGN, "%s: dense_out needs a 16-byte aligned base and row stride", fn);
        Range rd = range_of(dense, ((T - 1) * ldd + O) * es, "dense_out");
        if (overlap(rd, rin) || overlap(rd, rv) || overlap(rd, rm))
            return fail(NM_ERR_ALIAS, "%s: dense_out must not overlap g, vals or meta", fn);
    }
    return NM_OK;
}

// workspace of `need` bytes: present, large enough, aligned, and clear of dW and of every input range
int check_workspace(const char *fn, size_t need, const void *workspace, size_t workspace_bytes, const Range &rd,
                    const Range *inputs, int n_inputs)
{
    if (!need) return NM_OK;
    if (!workspace || workspace_bytes < need)
        return fail(NM_ERR_WORKSPACE, "%s: workspace of %zu bytes required, %zu given", fn, need, workspace ? workspace_bytes : (size_t)0);
    if (!aligned16(workspace)) return fail(NM_ERR_ALIGN, "%s: workspace needs a 16-byte aligned base", fn);
    const Range rw = range_of(workspace, (int64_t)need, "workspace");
    if (overlap(rw, rd)) return fail(NM_ERR_ALIAS, "%s: workspace must not overlap dW", fn);
    for (int i = 0; i < n_inputs; ++i)
        if (overlap(rw, inputs[i])) return fail(NM_ERR_ALIAS, "%s: workspace must not overlap %s", fn, inputs[i].name);
    return NM_OK;
}

int launched(const char *fn, hipError_t e)
{
    if (e != hipSuccess) return fail(NM_ERR_LAUNCH, "%s: HIP launch failed: %s", fn, hipGetErrorString(e));
    g_err[0] = 0;
    return NM_OK;
}

}  // namespace

extern "C" {

int mvue_prune_1of2(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype, uint64_t seed, uint32_t stream_id,
                    void *vals, uint16_t *meta, void *dense_out, int64_t ldd, void *hip_stream)
{
    const char *fn = "mvue_prune_1of2";
    if (int rc = check_tensor(fn, g, T, O, ldg, dtype, "g")) return rc;
    if (int rc = check_outputs(fn, g, T, O, ldg, dtype, vals, meta, dense_out, ldd)) return rc;
    return launched(fn, nm::launch_prune(dtype, 2, 0, g, T, O, ldg, seed, stream_id, vals, meta, dense_out, ldd,
                                         (hipStream_t)hip_stream));
}

int mvue_prune_2of4(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype, uint64_t seed, uint32_t stream_id,
                    int mode, void *vals, uint16_t *meta, void *dense_out, int64_t ldd, void *hip_stream)
{
    const char *fn = "mvue_prune_2of4";
    if (mode != 0 && mode != 1)
        return fail(NM_ERR_UNSUPPORTED, "%s: unknown mode %d (0 = optimal MVUE, 1 = approx-MVUE)", fn, mode);
    if (int rc = check_tensor(fn, g, T, O, ldg, dtype, "g")) return rc;
    if (int rc = check_outputs(fn, g, T, O, ldg, dtype, vals, meta, dense_out, ldd)) return rc;
    return launched(fn, nm::launch_prune(dtype, 4, mode, g, T, O, ldg, seed, stream_id, vals, meta, dense_out, ldd,
                                         (hipStream_t)hip_stream));
}

int mvue_prune_1of4(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype, uint64_t seed, uint32_t stream_id,
                    void *vals, uint16_t *meta, void *dense_out, int64_t ldd, void *hip_stream)
{
    const char *fn = "mvue_prune_1of4";
    if (int rc = check_tensor(fn, g, T, O, ldg, dtype, "g")) return rc;
    if (int rc = check_outputs(fn, g, T, O, ldg, dtype, vals, meta, dense_out, ldd)) return rc;
    return launched(fn, nm::launch_prune(dtype, 4, 2, g, T, O, ldg, seed, stream_id, vals, meta, dense_out, ldd,
                                         (hipStream_t)hip_stream));
}

int nm_prune_greedy(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype, int n, int m,
                    void *vals, uint16_t *meta, void *dense_out, int64_t ldd, void *hip_stream)
{
    const char *fn = "nm_prune_greedy";
    if (!((n == 1 && m == 2) || (n == 2 && m == 4)))
        return fail(NM_ERR_UNSUPPORTED, "%s: (n,m)=(%d,%d); only 1:2 and 2:4 exist in the group format", fn, n, m);
    if (int rc = check_tensor(fn, g, T, O, ldg, dtype, "g")) return rc;
    if (int rc = check_outputs(fn, g, T, O, ldg, dtype, vals, meta, dense_out, ldd)) return rc;
    return launched(fn, nm::launch_prune(dtype, m, 4, g, T, O, ldg, 0, 0, vals, meta, dense_out, ldd, (hipStream_t)hip_stream));
}

int mvue_prune_4of8_approx(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype, uint64_t seed, uint32_t stream_id,
                           void *vals, uint32_t *meta32, void *dense_out, int64_t ldd, void *hip_stream)
{
    const char *fn = "mvue_prune_4of8_approx";
    if (int rc = check_tensor(fn, g, T, O, ldg, dtype, "g")) return rc;
    if (T == 0 || O == 0) { g_err[0] = 0; return NM_OK; }
    if (!vals || !meta32) return fail(NM_ERR_NULL, "%s: vals and meta32 must not be NULL", fn);
    if (!aligned16(vals) || !aligned16(meta32)) return fail(NM_ERR_ALIGN, "%s: vals and meta32 need 16-byte aligned bases", fn);
    const int64_t es = esize(dtype);
    Range rin = range_of(g, ((T - 1) * ldg + O) * es, "g");
    Range rv = range_of(vals, T / 2 * O * es, "vals"), rm = range_of(meta32, T / 16 * O * 4, "meta32");
    if (overlap(rin, rv) || overlap(rin, rm) || overlap(rv, rm)) return fail(NM_ERR_ALIAS, "%s: g, vals and meta32 must not overlap", fn);
    if (dense_out) {
        if (ldd < O || too_big(T, ldd)) return fail(NM_ERR_SHAPE, "%s: ldd=%lld is smaller than O=%lld (or beyond 2^58 elements)", fn, (long long)ldd, (long long)O);
        if (!aligned16(dense_out) || (ldd * es) % 16) return fail(NM_ERR_ALIGN, "%s: dense_out needs a 16-byte aligned base and row stride", fn);
        Range rd = range_of(dense_out, ((T - 1) * ldd + O) * es, "dense_out");
        if (overlap(rd, rin) || overlap(rd, rv) || overlap(rd, rm)) return fail(NM_ERR_ALIAS, "%s: dense_out must not overlap g, vals or meta32", fn);
    }
    return launched(fn, nm::launch_prune_4of8_approx(dtype, g, T, O, ldg, seed, stream_id, vals, meta32, dense_out, ldd,
                                                     (hipStream_t)hip_stream));
}

static int prune_producer(const char *fn, int m, int est, const void *u, int64_t ldu, const void *d, int64_t ldd, int64_t T, int64_t O,
                          int dtype, uint64_t seed, uint32_t stream_id, void *g_out, int64_t ldg, void *vals, uint16_t *meta,
                          void *hip_stream)
{
    if (int rc = check_tensor(fn, u, T, O, ldu, dtype, "u")) return rc;
    if (int rc = check_tensor(fn, d, T, O, ldd, dtype, "d")) return rc;
    if (int rc = check_tensor(fn, g_out, T, O, ldg, dtype, "g_out")) return rc;
    if (T == 0 || O == 0) { g_err[0] = 0; return NM_OK; }
    if (!vals || !meta) return fail(NM_ERR_NULL, "%s: vals and meta must not be NULL", fn);
    if (!aligned16(vals) || !aligned16(meta)) return fail(NM_ERR_ALIGN, "%s: vals and meta need 16-byte aligned bases", fn);
    const int64_t es = esize(dtype);
    const Range ru = range_of(u, ((T - 1) * ldu + O) * es, "u"), rdd = range_of(d, ((T - 1) * ldd + O) * es, "d");
    const Range rg = range_of(g_out, ((T - 1) * ldg + O) * es, "g_out");
    const Range rv = range_of(vals, T / 2 * O * es, "vals"), rm = range_of(meta, T / 16 * O * 2, "meta");
    if (overlap(rg, ru) || overlap(rg, rdd) || overlap(rv, ru) || overlap(rv, rdd) || overlap(rm, ru) || overlap(rm, rdd) ||
        overlap(rg, rv) || overlap(rg, rm) || overlap(rv, rm))
        return fail(NM_ERR_ALIAS, "%s: g_out, vals and meta must not overlap each other or an input", fn);
    return launched(fn, nm::launch_prune_producer(dtype, m, est, u, ldu, d, ldd, T, O, seed, stream_id, g_out, ldg, vals, meta,
                                                  (hipStream_t)hip_stream));
}

int mvue_prune_2of4_producer(const void *u, int64_t ldu, const void *d, int64_t ldd, int64_t T, int64_t O, int dtype,
                             uint64_t seed, uint32_t stream_id, int mode, void *g_out, int64_t ldg, void *vals, uint16_t *meta,
                             void *hip_stream)
{
    if (mode != 0 && mode != 1)
        return fail(NM_ERR_UNSUPPORTED, "mvue_prune_2of4_producer: unknown mode %d (0 = optimal MVUE, 1 = approx-MVUE)", mode);
    return prune_producer("mvue_prune_2of4_producer", 4, mode, u, ldu, d, ldd, T, O, dtype, seed, stream_id, g_out, ldg, vals, meta,
                          hip_stream);
}

int mvue_prune_1of2_producer(const void *u, int64_t ldu, const void *d, int64_t ldd, int64_t T, int64_t O, int dtype,
                             uint64_t seed, uint32_t stream_id, void *g_out, int64_t ldg, void *vals, uint16_t *meta,
                             void *hip_stream)
{
    return prune_producer("mvue_prune_1of2_producer", 2, 0, u, ldu, d, ldd, T, O, dtype, seed, stream_id, g_out, ldg, vals, meta,
                          hip_stream);
}

static int prune_transposed(const char *fn, int est, const void *gT, int64_t T, int64_t O, int64_t ldt, int dtype, uint64_t seed,
                            uint32_t stream_id, void *vals, uint16_t *meta, void *hip_stream)
{
    if (dtype != NM_F32 && dtype != NM_BF16) return fail(NM_ERR_DTYPE, "%s: dtype %d is not NM_F32 (0) or NM_BF16 (1)", fn, dtype);
    if (T < 0 || O < 0) return fail(NM_ERR_SHAPE, "%s: negative size T=%lld O=%lld", fn, (long long)T, (long long)O);
    if (T % 16) return fail(NM_ERR_SHAPE, "%s: T=%lld is not a multiple of 16 (pad with zero tokens)", fn, (long long)T);
    if (O % 8) return fail(NM_ERR_SHAPE, "%s: O=%lld is not a multiple of 8 (pad with zero rows)", fn, (long long)O);
    if (too_big(O, T) || too_big(O, ldt)) return fail(NM_ERR_SHAPE, "%s: gT is larger than 2^58 elements", fn);
    if (T == 0 || O == 0) { g_err[0] = 0; return NM_OK; }
    if (!gT || !vals || !meta) return fail(NM_ERR_NULL, "%s: gT, vals and meta must not be NULL", fn);
    if (ldt < T) return fail(NM_ERR_SHAPE, "%s: row stride %lld of gT is smaller than T=%lld", fn, (long long)ldt, (long long)T);
    const int64_t es = esize(dtype);
    if (!aligned16(gT) || (ldt * es) % 16 || !aligned16(vals) || !aligned16(meta))
        return fail(NM_ERR_ALIGN, "%s: gT (base and row stride), vals and meta need 16-byte alignment", fn);
    Range rin = range_of(gT, ((O - 1) * ldt + T) * es, "gT");
    Range rv = range_of(vals, T / 2 * O * es, "vals"), rm = range_of(meta, T / 16 * O * 2, "meta");
    if (overlap(rin, rv) || overlap(rin, rm) || overlap(rv, rm)) return fail(NM_ERR_ALIAS, "%s: gT, vals and meta must not overlap", fn);
    return launched(fn, nm::launch_prune_transposed(dtype, est, gT, T, O, ldt, seed, stream_id, vals, meta, (hipStream_t)hip_stream));
}

int mvue_prune_2of4_t(const void *gT, int64_t T, int64_t O, int64_t ldt, int dtype, uint64_t seed, uint32_t stream_id,
                      int mode, void *vals, uint16_t *meta, void *hip_stream)
{
    if (mode != 0 && mode != 1)
        return fail(NM_ERR_UNSUPPORTED, "mvue_prune_2of4_t: unknown mode %d (0 = optimal MVUE, 1 = approx-MVUE)", mode);
    return prune_transposed("mvue_prune_2of4_t", mode, gT, T, O, ldt, dtype, seed, stream_id, vals, meta, hip_stream);
}

int mvue_prune_1of2_t(const void *gT, int64_t T, int64_t O, int64_t ldt, int dtype, uint64_t seed, uint32_t stream_id,
                      void *vals, uint16_t *meta, void *hip_stream)
{
    return prune_transposed("mvue_prune_1of2_t", 3, gT, T, O, ldt, dtype, seed, stream_id, vals, meta, hip_stream);
}

int nm_compress(const void *dense, int64_t T, int64_t O, int64_t ld, int dtype, int n, int m, void *vals,
                uint16_t *meta, int32_t *bad_blocks, void *hip_stream)
{
    const char *fn = "nm_compress";
    if (!((n == 1 && m == 2) || (n == 2 && m == 4)))
        return fail(NM_ERR_UNSUPPORTED, "%s: (n,m)=(%d,%d); only 1:2 and 2:4 exist in the group format", fn, n, m);
    if (int rc = check_tensor(fn, dense, T, O, ld, dtype, "dense")) return rc;
    if (int rc = check_outputs(fn, dense, T, O, ld, dtype, vals, meta, nullptr, 0)) return rc;
    return launched(fn, nm::launch_compress(dtype, m, dense, T, O, ld, vals, meta, bad_blocks, (hipStream_t)hip_stream));
}

size_t nm_update_gemm_workspace(int64_t T, int64_t O, int64_t I, int dtype)
{
    if (T < 0 || O < 0 || I < 0 || (dtype != NM_F32 && dtype != NM_BF16 && dtype != NM_F32_BF16X3)) return 0;
    return nm::update_gemm_workspace(dtype, T, O, I);
}

// nm_update_gemm and nm_update_gemm_static: the same checks and kernels; the second takes its split-K workspace from
// the library's static device array instead of the caller
static int update_gemm_checked(const char *fn, bool static_scratch, const void *vals, const uint16_t *meta, const void *h,
                               int64_t ldh, float *dW, int64_t lddw, int64_t T, int64_t O, int64_t I, int dtype, float beta,
                               void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (dtype != NM_F32 && dtype != NM_BF16 && dtype != NM_F32_BF16X3)
        return fail(NM_ERR_DTYPE, "%s: dtype %d is not NM_F32 (0), NM_BF16 (1) or NM_F32_BF16X3 (2)", fn, dtype);
    if (T < 0 || O < 0 || I < 0) return fail(NM_ERR_SHAPE, "%s: negative size", fn);
    if (T % 16) return fail(NM_ERR_SHAPE, "%s: T=%lld is not a multiple of 16", fn, (long long)T);
    if (O % 8 || I % 8) return fail(NM_ERR_SHAPE, "%s: O=%lld and I=%lld must be multiples of 8", fn, (long long)O, (long long)I);
    if (too_big(T, O) || too_big(T, I) || too_big(T, ldh) || too_big(O, I) || too_big(O, lddw))
        return fail(NM_ERR_SHAPE, "%s: a tensor is larger than 2^58 elements", fn);
    if (!(beta == 0.0f || beta == 1.0f)) return fail(NM_ERR_UNSUPPORTED, "%s: beta must be 0 or 1", fn);
    if (O == 0 || I == 0) { g_err[0] = 0; return NM_OK; }
    const int64_t es = esize(dtype);
    if (!dW) return fail(NM_ERR_NULL, "%s: dW is NULL", fn);
    if (lddw < I) return fail(NM_ERR_SHAPE, "%s: lddw=%lld is smaller than I=%lld", fn, (long long)lddw, (long long)I);
    if (!aligned16(dW) || (lddw * 4) % 16) return fail(NM_ERR_ALIGN, "%s: dW needs a 16-byte aligned base and row stride", fn);
    Range rd = range_of(dW, ((O - 1) * lddw + I) * 4, "dW");
    Range rin[3];
    int n_in = 0;
    if (T > 0) {
        if (!vals || !meta || !h) return fail(NM_ERR_NULL, "%s: vals, meta and h must not be NULL", fn);
        if (ldh < I) return fail(NM_ERR_SHAPE, "%s: ldh=%lld is smaller than I=%lld", fn, (long long)ldh, (long long)I);
        // the kernels address a few hundred rows of h, and a few dozen token groups of vals, through 32-bit byte offsets
        if (ldh > (1 << 21) || O > (1 << 21))
            return fail(NM_ERR_UNSUPPORTED, "%s: O=%lld and ldh=%lld must not exceed 2^21", fn, (long long)O, (long long)ldh);
        if (!aligned16(vals) || !aligned16(meta) || !aligned16(h) || (ldh * es) % 16)
            return fail(NM_ERR_ALIGN, "%s: vals, meta, h need 16-byte aligned bases (and h a 16-byte row stride)", fn);
        rin[0] = range_of(vals, T / 2 * O * es, "vals"); rin[1] = range_of(meta, T / 16 * O * 2, "meta");
        rin[2] = range_of(h, ((T - 1) * ldh + I) * es, "h");
        n_in = 3;
        if (overlap(rd, rin[0]) || overlap(rd, rin[1]) || overlap(rd, rin[2])) return fail(NM_ERR_ALIAS, "%s: dW must not overlap an input", fn);
    }
    const size_t need = nm::update_gemm_workspace(dtype, T, O, I);
    if (static_scratch) {
        workspace = nullptr;
        workspace_bytes = 0;
        if (need > nm::static_scratch_bytes())
            return fail(NM_ERR_WORKSPACE, "%s: this problem needs %zu bytes of split-K scratch, the static array holds %zu; "
                        "use nm_update_gemm with a workspace", fn, need, nm::static_scratch_bytes());
        if (need) {
            const hipError_t e = nm::static_scratch(&workspace);
            if (e != hipSuccess) return fail(NM_ERR_LAUNCH, "%s: address of the static scratch array: %s", fn, hipGetErrorString(e));
            workspace_bytes = nm::static_scratch_bytes();
        }
    } else if (int rc = check_workspace(fn, need, workspace, workspace_bytes, rd, rin, n_in)) return rc;
    return launched(fn, nm::launch_update_gemm(dtype, vals, meta, h, ldh, dW, lddw, T, O, I, beta, workspace,
                                               workspace_bytes, (hipStream_t)hip_stream));
}

int nm_update_gemm(const void *vals, const uint16_t *meta, const void *h, int64_t ldh, float *dW, int64_t lddw,
                   int64_t T, int64_t O, int64_t I, int dtype, float beta, void *workspace, size_t workspace_bytes,
                   void *hip_stream)
{
    return update_gemm_checked("nm_update_gemm", false, vals, meta, h, ldh, dW, lddw, T, O, I, dtype, beta, workspace,
                               workspace_bytes, hip_stream);
}

int nm_update_gemm_static(const void *vals, const uint16_t *meta, const void *h, int64_t ldh, float *dW, int64_t lddw,
                          int64_t T, int64_t O, int64_t I, int dtype, float beta, void *hip_stream)
{
    return update_gemm_checked("nm_update_gemm_static", true, vals, meta, h, ldh, dW, lddw, T, O, I, dtype, beta, nullptr, 0,
                               hip_stream);
}

size_t nm_update_gemm_static_max(void) { return nm::static_scratch_bytes(); }

size_t nm_update_gemm_shifted_workspace(int64_t T, int64_t O, int64_t cb, int n_shift)
{
    if (T < 0 || O < 0 || cb < 0 || n_shift < 1 || n_shift > 32) return 0;
    return nm::update_gemm_smfmac_shifted_workspace(T, O, cb * n_shift);
}

int nm_update_gemm_shifted(const void *vals, const uint16_t *meta, const void *x, int64_t ldx, int64_t cb,
                           const int64_t *row_shift, int n_shift, float *dW, int64_t lddw, int64_t T, int64_t O,
                           int dtype, float beta, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const char *fn = "nm_update_gemm_shifted";
    if (dtype != NM_F32 && dtype != NM_BF16) return fail(NM_ERR_DTYPE, "%s: dtype %d is not NM_F32 (0) or NM_BF16 (1)", fn, dtype);
    if (dtype != NM_BF16) return fail(NM_ERR_UNSUPPORTED, "%s: only NM_BF16 operands (the sparse-MFMA kernels) take shifted views", fn);
    if (T < 0 || O < 0 || cb < 0) return fail(NM_ERR_SHAPE, "%s: negative size", fn);
    if (n_shift < 1 || n_shift > 32) return fail(NM_ERR_SHAPE, "%s: n_shift=%d must be 1..32", fn, n_shift);
    if (!row_shift) return fail(NM_ERR_NULL, "%s: row_shift is NULL", fn);
    if (T % 16) return fail(NM_ERR_SHAPE, "%s: T=%lld is not a multiple of 16", fn, (long long)T);
    if (O % 8 || cb % 8) return fail(NM_ERR_SHAPE, "%s: O=%lld and cb=%lld must be multiples of 8", fn, (long long)O, (long long)cb);
    if (too_big(T, O) || too_big(T + 64, 32 * cb) || too_big(T + 64, ldx) || too_big(O, 32 * cb) || too_big(O, lddw))
        return fail(NM_ERR_SHAPE, "%s: a tensor is larger than 2^58 elements", fn);
    if (!(beta == 0.0f || beta == 1.0f)) return fail(NM_ERR_UNSUPPORTED, "%s: beta must be 0 or 1", fn);
    const int64_t I = cb * n_shift;
    if (O == 0 || I == 0) { g_err[0] = 0; return NM_OK; }
    int64_t margin = 0;
    for (int j = 0; j < n_shift; ++j) margin = row_shift[j] < -margin ? -row_shift[j] : row_shift[j] > margin ? row_shift[j] : margin;
    if (margin > (1 << 20)) return fail(NM_ERR_UNSUPPORTED, "%s: row shifts must not exceed 2^20 rows", fn);
    if (!dW) return fail(NM_ERR_NULL, "%s: dW is NULL", fn);
    if (lddw < I) return fail(NM_ERR_SHAPE, "%s: lddw=%lld is smaller than I=%lld", fn, (long long)lddw, (long long)I);
    if (!aligned16(dW) || (lddw * 4) % 16) return fail(NM_ERR_ALIGN, "%s: dW needs a 16-byte aligned base and row stride", fn);
    Range rd = range_of(dW, ((O - 1) * lddw + I) * 4, "dW");
    Range rin[3];
    int n_in = 0;
    if (T > 0) {
        if (!vals || !meta || !x) return fail(NM_ERR_NULL, "%s: vals, meta and x must not be NULL", fn);
        if (ldx < cb) return fail(NM_ERR_SHAPE, "%s: ldx=%lld is smaller than cb=%lld", fn, (long long)ldx, (long long)cb);
        if (ldx > (1 << 21) || O > (1 << 21) || (margin + 512) * ldx > (1ll << 30))
            return fail(NM_ERR_UNSUPPORTED, "%s: O, ldx and (shift x ldx) exceed what 32-bit byte offsets reach", fn);
        if (!aligned16(vals) || !aligned16(meta) || !aligned16(x) || (ldx * 2) % 16)
            return fail(NM_ERR_ALIGN, "%s: vals, meta, x need 16-byte aligned bases (and x a 16-byte row stride)", fn);
        rin[0] = range_of(vals, T / 2 * O * 2, "vals"); rin[1] = range_of(meta, T / 16 * O * 2, "meta");
        rin[2] = range_of((const char *)x - margin * ldx * 2, ((T + 2 * margin - 1) * ldx + cb) * 2, "x");
        n_in = 3;
        if (overlap(rd, rin[0]) || overlap(rd, rin[1]) || overlap(rd, rin[2])) return fail(NM_ERR_ALIAS, "%s: dW must not overlap an input", fn);
    }
    if (int rc = check_workspace(fn, nm::update_gemm_smfmac_shifted_workspace(T, O, I), workspace, workspace_bytes, rd, rin, n_in)) return rc;
    return launched(fn, nm::launch_update_gemm_smfmac_shifted(vals, meta, x, ldx, cb, row_shift, n_shift, dW, lddw, T, O, beta,
                                                              workspace, (hipStream_t)hip_stream));
}

static int prune_q8(const char *fn, int est, const void *g, int64_t T, int64_t O, int64_t ldg, int dtype, uint64_t seed,
                    uint32_t stream_id, float scale, const float *scale_dev, bool device_scale, uint8_t *vals8, uint32_t *meta32,
                    void *hip_stream)
{
    if (int rc = check_tensor(fn, g, T, O, ldg, dtype, "g")) return rc;
    if (T % 32) return fail(NM_ERR_SHAPE, "%s: T=%lld is not a multiple of 32 (pad with zero rows)", fn, (long long)T);
    if (device_scale) {
        if (!scale_dev) return fail(NM_ERR_NULL, "%s: the scale record is NULL", fn);
        if (!aligned16(scale_dev)) return fail(NM_ERR_ALIGN, "%s: the scale record needs a 16-byte aligned base", fn);
    } else if (!(scale > 0.0f) || !(scale < __builtin_inff())) return fail(NM_ERR_SHAPE, "%s: scale must be positive and finite", fn);
    if (T == 0 || O == 0) { g_err[0] = 0; return NM_OK; }
    if (!vals8 || !meta32) return fail(NM_ERR_NULL, "%s: vals8 and meta32 must not be NULL", fn);
    if (!aligned16(vals8) || !aligned16(meta32)) return fail(NM_ERR_ALIGN, "%s: vals8 and meta32 need 16-byte aligned bases", fn);
    Range rin = range_of(g, ((T - 1) * ldg + O) * esize(dtype), "g");
    Range rv = range_of(vals8, T / 2 * O, "vals8"), rm = range_of(meta32, T / 32 * O * 4, "meta32");
    if (overlap(rin, rv) || overlap(rin, rm) || overlap(rv, rm))
        return fail(NM_ERR_ALIAS, "%s: g, vals8 and meta32 must not overlap", fn);
    if (device_scale) {
        Range rs = range_of(scale_dev, 16, "scale record");
        if (overlap(rs, rv) || overlap(rs, rm)) return fail(NM_ERR_ALIAS, "%s: the scale record must not overlap an output", fn);
    }
    return launched(fn, nm::launch_prune_q8(dtype, est, g, T, O, ldg, seed, stream_id, scale, device_scale ? scale_dev : nullptr,
                                            vals8, meta32, (hipStream_t)hip_stream));
}

static int prune_q8_transposed(const char *fn, int est, const void *gT, int64_t T, int64_t O, int64_t ldt, int dtype, uint64_t seed,
                               uint32_t stream_id, float scale, const float *scale_rec, uint8_t *vals8, uint32_t *meta32,
                               void *hip_stream)
{
    if (dtype != NM_F32 && dtype != NM_BF16) return fail(NM_ERR_DTYPE, "%s: dtype %d is not NM_F32 (0) or NM_BF16 (1)", fn, dtype);
    if (T < 0 || O < 0) return fail(NM_ERR_SHAPE, "%s: negative size T=%lld O=%lld", fn, (long long)T, (long long)O);
    if (T % 32) return fail(NM_ERR_SHAPE, "%s: T=%lld is not a multiple of 32 (pad with zero tokens)", fn, (long long)T);
    if (O % 8) return fail(NM_ERR_SHAPE, "%s: O=%lld is not a multiple of 8 (pad with zero rows)", fn, (long long)O);
    if (too_big(O, T) || too_big(O, ldt)) return fail(NM_ERR_SHAPE, "%s: gT is larger than 2^58 elements", fn);
    if (scale_rec) {
        if (!aligned16(scale_rec)) return fail(NM_ERR_ALIGN, "%s: the scale record needs a 16-byte aligned base", fn);
    } else if (!(scale > 0.0f) || !(scale < __builtin_inff())) return fail(NM_ERR_SHAPE, "%s: scale must be positive and finite", fn);
    if (T == 0 || O == 0) { g_err[0] = 0; return NM_OK; }
    if (!gT || !vals8 || !meta32) return fail(NM_ERR_NULL, "%s: gT, vals8 and meta32 must not be NULL", fn);
    if (ldt < T) return fail(NM_ERR_SHAPE, "%s: row stride %lld of gT is smaller than T=%lld", fn, (long long)ldt, (long long)T);
    const int64_t es = esize(dtype);
    if (!aligned16(gT) || (ldt * es) % 16 || !aligned16(vals8) || !aligned16(meta32))
        return fail(NM_ERR_ALIGN, "%s: gT (base and row stride), vals8 and meta32 need 16-byte alignment", fn);
    Range rin = range_of(gT, ((O - 1) * ldt + T) * es, "gT");
    Range rv = range_of(vals8, T / 2 * O, "vals8"), rm = range_of(meta32, T / 32 * O * 4, "meta32");
    if (overlap(rin, rv) || overlap(rin, rm) || overlap(rv, rm)) return fail(NM_ERR_ALIAS, "%s: gT, vals8 and meta32 must not overlap", fn);
    if (scale_rec) {
        Range rs = range_of(scale_rec, 16, "scale record");
        if (overlap(rs, rv) || overlap(rs, rm)) return fail(NM_ERR_ALIAS, "%s: the scale record must not overlap an output", fn);
    }
    return launched(fn, nm::launch_prune_q8_transposed(dtype, est, gT, T, O, ldt, seed, stream_id, scale_rec ? 1.0f : scale, scale_rec,
                                                       vals8, meta32, (hipStream_t)hip_stream));
}

int mvue_prune_2of4_q8_t(const void *gT, int64_t T, int64_t O, int64_t ldt, int dtype, uint64_t seed, uint32_t stream_id, int mode,
                         float scale, const float *scale_rec, uint8_t *vals8, uint32_t *meta32, void *hip_stream)
{
    if (mode != 0 && mode != 1)
        return fail(NM_ERR_UNSUPPORTED, "mvue_prune_2of4_q8_t: unknown mode %d (0 = optimal MVUE, 1 = approx-MVUE)", mode);
    return prune_q8_transposed("mvue_prune_2of4_q8_t", mode, gT, T, O, ldt, dtype, seed, stream_id, scale, scale_rec, vals8, meta32,
                               hip_stream);
}

int mvue_prune_1of2_q8_t(const void *gT, int64_t T, int64_t O, int64_t ldt, int dtype, uint64_t seed, uint32_t stream_id, float scale,
                         const float *scale_rec, uint8_t *vals8, uint32_t *meta32, void *hip_stream)
{
    return prune_q8_transposed("mvue_prune_1of2_q8_t", 3, gT, T, O, ldt, dtype, seed, stream_id, scale, scale_rec, vals8, meta32,
                               hip_stream);
}

int mvue_prune_2of4_q8(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype, uint64_t seed, uint32_t stream_id,
                       int mode, float scale, uint8_t *vals8, uint32_t *meta32, void *hip_stream)
{
    if (mode != 0 && mode != 1)
        return fail(NM_ERR_UNSUPPORTED, "mvue_prune_2of4_q8: unknown mode %d (0 = optimal MVUE, 1 = approx-MVUE)", mode);
    return prune_q8("mvue_prune_2of4_q8", mode, g, T, O, ldg, dtype, seed, stream_id, scale, nullptr, false, vals8, meta32, hip_stream);
}

int mvue_prune_2of4_q8_ds(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype, uint64_t seed, uint32_t stream_id,
                          int mode, const float *scale_rec, uint8_t *vals8, uint32_t *meta32, void *hip_stream)
{
    if (mode != 0 && mode != 1)
        return fail(NM_ERR_UNSUPPORTED, "mvue_prune_2of4_q8_ds: unknown mode %d (0 = optimal MVUE, 1 = approx-MVUE)", mode);
    return prune_q8("mvue_prune_2of4_q8_ds", mode, g, T, O, ldg, dtype, seed, stream_id, 1.0f, scale_rec, true, vals8, meta32, hip_stream);
}

int mvue_prune_1of2_q8_ds(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype, uint64_t seed, uint32_t stream_id,
                          const float *scale_rec, uint8_t *vals8, uint32_t *meta32, void *hip_stream)
{
    return prune_q8("mvue_prune_1of2_q8_ds", 3, g, T, O, ldg, dtype, seed, stream_id, 1.0f, scale_rec, true, vals8, meta32, hip_stream);
}

int nm_q8_scale(const void *t, int64_t R, int64_t C, int64_t ld, int dtype, float top, float *scale_rec, void *hip_stream)
{
    const char *fn = "nm_q8_scale";
    if (dtype != NM_F32 && dtype != NM_BF16) return fail(NM_ERR_DTYPE, "%s: dtype %d is not NM_F32 (0) or NM_BF16 (1)", fn, dtype);
    if (R < 0 || C < 0) return fail(NM_ERR_SHAPE, "%s: negative size", fn);
    if (C % 8) return fail(NM_ERR_SHAPE, "%s: C=%lld is not a multiple of 8", fn, (long long)C);
    if (too_big(R, C) || too_big(R, ld)) return fail(NM_ERR_SHAPE, "%s: the tensor is larger than 2^58 elements", fn);
    if (!(top > 0.0f) || !(top < __builtin_inff())) return fail(NM_ERR_SHAPE, "%s: top must be positive and finite", fn);
    if (!scale_rec) return fail(NM_ERR_NULL, "%s: the scale record is NULL", fn);
    if (!aligned16(scale_rec)) return fail(NM_ERR_ALIGN, "%s: the scale record needs a 16-byte aligned base", fn);
    if (R > 0 && C > 0) {
        if (!t) return fail(NM_ERR_NULL, "%s: t is NULL", fn);
        if (ld < C) return fail(NM_ERR_SHAPE, "%s: row stride %lld is smaller than C=%lld", fn, (long long)ld, (long long)C);
        if (!aligned16(t) || (ld * esize(dtype)) % 16) return fail(NM_ERR_ALIGN, "%s: t needs a 16-byte aligned base and row stride", fn);
        if (overlap(range_of(t, ((R - 1) * ld + C) * esize(dtype), "t"), range_of(scale_rec, 16, "scale record")))
            return fail(NM_ERR_ALIAS, "%s: the scale record must not overlap t", fn);
    }
    return launched(fn, nm::launch_q8_scale(dtype, t, R, C, ld, top, scale_rec, (hipStream_t)hip_stream));
}

int nm_rw_mix_probe(const void *src, void *dst, int64_t n_blocks, void *hip_stream)
{
    const char *fn = "nm_rw_mix_probe";
    if (n_blocks < 0) return fail(NM_ERR_SHAPE, "%s: negative size", fn);
    if (n_blocks > 0x7fffffffll) return fail(NM_ERR_SHAPE, "%s: more than 2^31 - 1 blocks", fn);
    if (n_blocks == 0) { g_err[0] = 0; return NM_OK; }
    if (!src || !dst) return fail(NM_ERR_NULL, "%s: src and dst must not be NULL", fn);
    if (!aligned16(src) || !aligned16(dst)) return fail(NM_ERR_ALIGN, "%s: src and dst need 16-byte alignment", fn);
    if (overlap(range_of(src, n_blocks * 65536, "src"), range_of(dst, n_blocks * 36864, "dst")))
        return fail(NM_ERR_ALIAS, "%s: dst must not overlap src", fn);
    return launched(fn, nm::launch_rw_mix_probe(src, dst, n_blocks, (hipStream_t)hip_stream));
}

int nm_cast_e4m3(const void *h, int64_t R, int64_t C, int64_t ld, int dtype, const float *scale_rec, uint8_t *h8, int64_t ld8,
                 void *hip_stream)
{
    const char *fn = "nm_cast_e4m3";
    if (dtype != NM_F32 && dtype != NM_BF16) return fail(NM_ERR_DTYPE, "%s: dtype %d is not NM_F32 (0) or NM_BF16 (1)", fn, dtype);
    if (R < 0 || C < 0) return fail(NM_ERR_SHAPE, "%s: negative size", fn);
    if (C % 16) return fail(NM_ERR_SHAPE, "%s: C=%lld is not a multiple of 16", fn, (long long)C);
    if (too_big(R, C) || too_big(R, ld) || too_big(R, ld8)) return fail(NM_ERR_SHAPE, "%s: a tensor is larger than 2^58 elements", fn);
    if (R == 0 || C == 0) { g_err[0] = 0; return NM_OK; }
    if (!h || !h8 || !scale_rec) return fail(NM_ERR_NULL, "%s: h, h8 and the scale record must not be NULL", fn);
    if (ld < C || ld8 < C) return fail(NM_ERR_SHAPE, "%s: a row stride is smaller than C=%lld", fn, (long long)C);
    if (!aligned16(h) || (ld * esize(dtype)) % 16 || !aligned16(h8) || ld8 % 16 || !aligned16(scale_rec))
        return fail(NM_ERR_ALIGN, "%s: h, h8 (bases and row strides) and the scale record need 16-byte alignment", fn);
    Range rh = range_of(h, ((R - 1) * ld + C) * esize(dtype), "h"), r8 = range_of(h8, (R - 1) * ld8 + C, "h8");
    Range rs = range_of(scale_rec, 16, "scale record");
    if (overlap(rh, r8) || overlap(rs, r8)) return fail(NM_ERR_ALIAS, "%s: h8 must not overlap h or the scale record", fn);
    return launched(fn, nm::launch_cast_e4m3(dtype, h, R, C, ld, scale_rec, h8, ld8, (hipStream_t)hip_stream));
}

int mvue_prune_1of2_q8(const void *g, int64_t T, int64_t O, int64_t ldg, int dtype, uint64_t seed, uint32_t stream_id,
                       float scale, uint8_t *vals8, uint32_t *meta32, void *hip_stream)
{
    return prune_q8("mvue_prune_1of2_q8", 3, g, T, O, ldg, dtype, seed, stream_id, scale, nullptr, false, vals8, meta32, hip_stream);
}

size_t nm_update_gemm_q8_workspace(int64_t T, int64_t O, int64_t I)
{
    if (T < 0 || O < 0 || I < 0) return 0;
    return nm::update_gemm_q8_workspace(T, O, I);
}

// scale records of the _ds entry points: present, aligned, clear of the output
static int check_scale_recs(const char *fn, const float *a, const float *b, const Range &rd)
{
    if (!a || !b) return fail(NM_ERR_NULL, "%s: a scale record is NULL", fn);
    if (!aligned16(a) || !aligned16(b)) return fail(NM_ERR_ALIGN, "%s: the scale records need 16-byte aligned bases", fn);
    if (overlap(range_of(a, 16, "scale record"), rd) || overlap(range_of(b, 16, "scale record"), rd))
        return fail(NM_ERR_ALIAS, "%s: dW must not overlap a scale record", fn);
    return NM_OK;
}

static int update_gemm_q8_checked(const char *fn, const uint8_t *vals8, const uint32_t *meta32, const uint8_t *h8, int64_t ldh,
                                  float *dW, int64_t lddw, int64_t T, int64_t O, int64_t I, nm::AlphaArg alpha, bool device_scale,
                                  float beta, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (T < 0 || O < 0 || I < 0) return fail(NM_ERR_SHAPE, "%s: negative size", fn);
    if (T % 32) return fail(NM_ERR_SHAPE, "%s: T=%lld is not a multiple of 32", fn, (long long)T);
    if (O % 8 || I % 16) return fail(NM_ERR_SHAPE, "%s: O=%lld must be a multiple of 8 and I=%lld of 16", fn, (long long)O, (long long)I);
    if (too_big(T, O) || too_big(T, I) || too_big(T, ldh) || too_big(O, I) || too_big(O, lddw))
        return fail(NM_ERR_SHAPE, "%s: a tensor is larger than 2^58 elements", fn);
    if (!(beta == 0.0f || beta == 1.0f)) return fail(NM_ERR_UNSUPPORTED, "%s: beta must be 0 or 1", fn);
    if (O == 0 || I == 0) { g_err[0] = 0; return NM_OK; }
    if (!dW) return fail(NM_ERR_NULL, "%s: dW is NULL", fn);
    if (lddw < I) return fail(NM_ERR_SHAPE, "%s: lddw=%lld is smaller than I=%lld", fn, (long long)lddw, (long long)I);
    if (!aligned16(dW) || (lddw * 4) % 16) return fail(NM_ERR_ALIGN, "%s: dW needs a 16-byte aligned base and row stride", fn);
    Range rd = range_of(dW, ((O - 1) * lddw + I) * 4, "dW");
    Range rin[3];
    int n_in = 0;
    if (T > 0) {
        if (!vals8 || !meta32 || !h8) return fail(NM_ERR_NULL, "%s: vals8, meta32 and h8 must not be NULL", fn);
        if (ldh < I) return fail(NM_ERR_SHAPE, "%s: ldh=%lld is smaller than I=%lld", fn, (long long)ldh, (long long)I);
        if (ldh > (1 << 21) || O > (1 << 21))
            return fail(NM_ERR_UNSUPPORTED, "%s: O=%lld and ldh=%lld must not exceed 2^21", fn, (long long)O, (long long)ldh);
        if (!aligned16(vals8) || !aligned16(meta32) || !aligned16(h8) || ldh % 16)
            return fail(NM_ERR_ALIGN, "%s: vals8, meta32, h8 need 16-byte aligned bases (and h8 a 16-byte row stride)", fn);
        rin[0] = range_of(vals8, T / 2 * O, "vals8"); rin[1] = range_of(meta32, T / 32 * O * 4, "meta32");
        rin[2] = range_of(h8, (T - 1) * ldh + I, "h8");
        n_in = 3;
        if (overlap(rd, rin[0]) || overlap(rd, rin[1]) || overlap(rd, rin[2])) return fail(NM_ERR_ALIAS, "%s: dW must not overlap an input", fn);
    }
    if (int rc = check_workspace(fn, nm::update_gemm_q8_workspace(T, O, I), workspace, workspace_bytes, rd, rin, n_in)) return rc;
    if (device_scale) if (int rc = check_scale_recs(fn, alpha.inv_a, alpha.inv_b, rd)) return rc;
    return launched(fn, nm::launch_update_gemm_q8(vals8, meta32, h8, ldh, dW, lddw, T, O, I, alpha, beta, workspace,
                                                  (hipStream_t)hip_stream));
}

int nm_update_gemm_q8(const uint8_t *vals8, const uint32_t *meta32, const uint8_t *h8, int64_t ldh, float *dW, int64_t lddw,
                      int64_t T, int64_t O, int64_t I, float alpha, float beta, void *workspace, size_t workspace_bytes,
                      void *hip_stream)
{
    return update_gemm_q8_checked("nm_update_gemm_q8", vals8, meta32, h8, ldh, dW, lddw, T, O, I, nm::AlphaArg(alpha), false, beta,
                                  workspace, workspace_bytes, hip_stream);
}

int nm_update_gemm_q8_ds(const uint8_t *vals8, const uint32_t *meta32, const uint8_t *h8, int64_t ldh, float *dW, int64_t lddw,
                         int64_t T, int64_t O, int64_t I, const float *scale_rec_g, float *scale_rec_h, float beta,
                         void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return update_gemm_q8_checked("nm_update_gemm_q8_ds", vals8, meta32, h8, ldh, dW, lddw, T, O, I,
                                  nm::AlphaArg(1.0f, scale_rec_g, scale_rec_h), true, beta, workspace, workspace_bytes, hip_stream);
}

size_t nm_update_gemm_q8_shifted_workspace(int64_t T, int64_t O, int64_t cb, int n_shift)
{
    if (T < 0 || O < 0 || cb < 0 || n_shift < 1 || n_shift > 32) return 0;
    return nm::update_gemm_q8_shifted_workspace(T, O, cb * n_shift);
}

static int update_gemm_q8_shifted_checked(const char *fn, const uint8_t *vals8, const uint32_t *meta32, const uint8_t *x8, int64_t ldx,
                                          int64_t cb, const int64_t *row_shift, int n_shift, float *dW, int64_t lddw, int64_t T,
                                          int64_t O, nm::AlphaArg alpha, bool device_scale, float beta, void *workspace,
                                          size_t workspace_bytes, void *hip_stream)
{
    if (T < 0 || O < 0 || cb < 0) return fail(NM_ERR_SHAPE, "%s: negative size", fn);
    if (n_shift < 1 || n_shift > 32) return fail(NM_ERR_SHAPE, "%s: n_shift=%d must be 1..32", fn, n_shift);
    if (!row_shift) return fail(NM_ERR_NULL, "%s: row_shift is NULL", fn);
    if (T % 32) return fail(NM_ERR_SHAPE, "%s: T=%lld is not a multiple of 32", fn, (long long)T);
    if (O % 8 || cb % 16) return fail(NM_ERR_SHAPE, "%s: O=%lld must be a multiple of 8 and cb=%lld of 16", fn, (long long)O, (long long)cb);
    if (too_big(T, O) || too_big(T + 64, 32 * cb) || too_big(T + 64, ldx) || too_big(O, 32 * cb) || too_big(O, lddw))
        return fail(NM_ERR_SHAPE, "%s: a tensor is larger than 2^58 elements", fn);
    if (!(beta == 0.0f || beta == 1.0f)) return fail(NM_ERR_UNSUPPORTED, "%s: beta must be 0 or 1", fn);
    const int64_t I = cb * n_shift;
    if (O == 0 || I == 0) { g_err[0] = 0; return NM_OK; }
    int64_t margin = 0;
    for (int j = 0; j < n_shift; ++j) margin = row_shift[j] < -margin ? -row_shift[j] : row_shift[j] > margin ? row_shift[j] : margin;
    if (margin > (1 << 20)) return fail(NM_ERR_UNSUPPORTED, "%s: row shifts must not exceed 2^20 rows", fn);
    if (!dW) return fail(NM_ERR_NULL, "%s: dW is NULL", fn);
    if (lddw < I) return fail(NM_ERR_SHAPE, "%s: lddw=%lld is smaller than I=%lld", fn, (long long)lddw, (long long)I);
    if (!aligned16(dW) || (lddw * 4) % 16) return fail(NM_ERR_ALIGN, "%s: dW needs a 16-byte aligned base and row stride", fn);
    Range rd = range_of(dW, ((O - 1) * lddw + I) * 4, "dW");
    Range rin[3];
    int n_in = 0;
    if (T > 0) {
        if (!vals8 || !meta32 || !x8) return fail(NM_ERR_NULL, "%s: vals8, meta32 and x8 must not be NULL", fn);
        if (ldx < cb) return fail(NM_ERR_SHAPE, "%s: ldx=%lld is smaller than cb=%lld", fn, (long long)ldx, (long long)cb);
        if (ldx > (1 << 21) || O > (1 << 21) || (margin + 1024) * ldx > (1ll << 30))
            return fail(NM_ERR_UNSUPPORTED, "%s: O, ldx and (shift x ldx) exceed what 32-bit byte offsets reach", fn);
        if (!aligned16(vals8) || !aligned16(meta32) || !aligned16(x8) || ldx % 16)
            return fail(NM_ERR_ALIGN, "%s: vals8, meta32, x8 need 16-byte aligned bases (and x8 a 16-byte row stride)", fn);
        rin[0] = range_of(vals8, T / 2 * O, "vals8"); rin[1] = range_of(meta32, T / 32 * O * 4, "meta32");
        rin[2] = range_of((const char *)x8 - margin * ldx, (T + 2 * margin - 1) * ldx + cb, "x8");
        n_in = 3;
        if (overlap(rd, rin[0]) || overlap(rd, rin[1]) || overlap(rd, rin[2])) return fail(NM_ERR_ALIAS, "%s: dW must not overlap an input", fn);
    }
    if (int rc = check_workspace(fn, nm::update_gemm_q8_shifted_workspace(T, O, I), workspace, workspace_bytes, rd, rin, n_in)) return rc;
    if (device_scale) if (int rc = check_scale_recs(fn, alpha.inv_a, alpha.inv_b, rd)) return rc;
    return launched(fn, nm::launch_update_gemm_q8_shifted(vals8, meta32, x8, ldx, cb, row_shift, n_shift, dW, lddw, T, O, alpha,
                                                          beta, workspace, (hipStream_t)hip_stream));
}

int nm_update_gemm_q8_shifted(const uint8_t *vals8, const uint32_t *meta32, const uint8_t *x8, int64_t ldx, int64_t cb,
                              const int64_t *row_shift, int n_shift, float *dW, int64_t lddw, int64_t T, int64_t O,
                              float alpha, float beta, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return update_gemm_q8_shifted_checked("nm_update_gemm_q8_shifted", vals8, meta32, x8, ldx, cb, row_shift, n_shift, dW, lddw, T, O,
                                          nm::AlphaArg(alpha), false, beta, workspace, workspace_bytes, hip_stream);
}

int nm_update_gemm_q8_shifted_ds(const uint8_t *vals8, const uint32_t *meta32, const uint8_t *x8, int64_t ldx, int64_t cb,
                                 const int64_t *row_shift, int n_shift, float *dW, int64_t lddw, int64_t T, int64_t O,
                                 const float *scale_rec_g, float *scale_rec_x, float beta, void *workspace,
                                 size_t workspace_bytes, void *hip_stream)
{
    return update_gemm_q8_shifted_checked("nm_update_gemm_q8_shifted_ds", vals8, meta32, x8, ldx, cb, row_shift, n_shift, dW, lddw, T, O,
                                          nm::AlphaArg(1.0f, scale_rec_g, scale_rec_x), true, beta, workspace, workspace_bytes,
                                          hip_stream);
}

const char *nm_last_error(void) { return g_err; }

const char *nm_version(void) { return "nm_mvue 0.1 gfx950"; }

}  // extern "C"
