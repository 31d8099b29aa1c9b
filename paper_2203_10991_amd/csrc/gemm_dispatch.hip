// Dtype dispatch of the update GEMM (eq. (3)) over the kernels of this library.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"

namespace nm {

size_t update_gemm_workspace(int dt, int64_t T, int64_t O, int64_t I)
{
    if (dt == NM_DT_F32_BF16X3) return update_gemm_f32_split_workspace(T, O, I);
    return dt == NM_DT_BF16 ? update_gemm_smfmac_workspace(T, O, I) : update_gemm_f32_workspace(T, O, I);
}

hipError_t launch_update_gemm(int dt, const void *vals, const uint16_t *meta, const void *h, int64_t ldh,
                              float *dW, int64_t lddw, int64_t T, int64_t O, int64_t I, float beta,
                              void *workspace, size_t workspace_bytes, hipStream_t st)
{
    (void)workspace_bytes;
    // bf16: 4:2 sparse MFMA.  binary32: gfx950's sparse matrix instructions take 16- and 8-bit operands only,
    // so the operand is expanded on its way into LDS and multiplied on the dense fp32 MFMA path.
    // binary32 as three bf16 terms: the six partial products as one run of the sparse 16-bit kernels.
    if (dt == NM_DT_F32_BF16X3) return launch_update_gemm_f32_split(vals, meta, h, ldh, dW, lddw, T, O, I, beta, workspace, st);
    if (dt == NM_DT_BF16) return launch_update_gemm_smfmac(vals, meta, h, ldh, dW, lddw, T, O, I, beta, workspace, st);
    return launch_update_gemm_f32(vals, meta, h, ldh, dW, lddw, T, O, I, beta, workspace, st);
}

}  // namespace nm
