// qg_gemm_small: placeholder until the matrix-core kernel lands.
#include "qg_common.h"

size_t qg_gemm_workspace_bytes(const QgLayout &L, int M)
{
    (void)L; (void)M;
    return QG_SECTION_ALIGN;
}

extern "C" int qg_gemm_small(const void *, int64_t, int64_t, int, int, const float *, int, float *,
                             void *, size_t, void *)
{
    return QG_ERR_UNSUPPORTED;
}
