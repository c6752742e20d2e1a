// Matrix-core variable-length attention (placeholder until the MFMA kernels land: reports
// "not supported" so that the scalar kernels are used).
#include "attention.h"

bool attn_mfma_supported(int) { return false; }
ms_status attn_mfma_forward(int, int, int, int, int, int, int, const int *, const void *, void *, float *, hipStream_t) {
    return ms_fail(MS_ERR_UNSUPPORTED, "attention: matrix-core path not built");
}
size_t attn_mfma_backward_scratch_bytes(int, int, int, int) { return 0; }
ms_status attn_mfma_backward(int, int, int, int, int, int, int, const int *, const void *, const void *, const float *,
                             const void *, void *, void *, hipStream_t) {
    return ms_fail(MS_ERR_UNSUPPORTED, "attention: matrix-core path not built");
}
