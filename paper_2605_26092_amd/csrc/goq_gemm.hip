// goq_gemm: many-token dual-PoT layer output (placeholder until the MFMA kernels land).
#include <hip/hip_runtime.h>
#include "goq_internal.h"

int goq_launch_gemm(hipStream_t, int, int, int64_t, int64_t, int64_t, const void *, const void *,
                    const float *, void *, int, int32_t *)
{
    return goq_set_error(GOQ_EUNSUPPORTED, "goq_gemm: not implemented yet");
}
