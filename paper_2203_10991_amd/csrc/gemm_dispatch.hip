// Shape/dtype dispatch of the update GEMM (eq. (3)) over the kernels of this library.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nm_internal.h"

namespace nm {

hipError_t launch_update_gemm_valu(int dt, const void *vals, const uint16_t *meta, const void *h, int64_t ldh,
                                   float *dW, int64_t lddw, int64_t T, int64_t O, int64_t I, float beta, hipStream_t st);
hipError_t launch_update_gemm_smfmac(const void *vals, const uint16_t *meta, const void *h, int64_t ldh, float *dW,
                                     int64_t lddw, int64_t T, int64_t O, int64_t I, float beta, void *workspace,
                                     hipStream_t st);
size_t update_gemm_smfmac_workspace(int64_t T, int64_t O, int64_t I);

size_t update_gemm_workspace(int dt, int64_t T, int64_t O, int64_t I)
{
    return dt == NM_DT_BF16 ? update_gemm_smfmac_workspace(T, O, I) : 0;
}

hipError_t launch_update_gemm(int dt, const void *vals, const uint16_t *meta, const void *h, int64_t ldh,
                              float *dW, int64_t lddw, int64_t T, int64_t O, int64_t I, float beta,
                              void *workspace, size_t workspace_bytes, hipStream_t st)
{
    (void)workspace_bytes;
    // bf16: sparse MFMA.  fp32: gfx950 has no sparse (nor any reduced-precision-free) matrix path for
    // binary32 inputs with 4:2 structure, so the operand is expanded on the fly on the vector ALU.
    if (dt == NM_DT_BF16 && T > 0)
        return launch_update_gemm_smfmac(vals, meta, h, ldh, dW, lddw, T, O, I, beta, workspace, st);
    return launch_update_gemm_valu(dt, vals, meta, h, ldh, dW, lddw, T, O, I, beta, st);
}

}  // namespace nm
