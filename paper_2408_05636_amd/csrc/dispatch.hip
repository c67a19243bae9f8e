// Shape-based choice between the kernel variants of one operation.
#include "common.h"

namespace sd {

hipError_t launch_linear(int dtype, const void* x, const void* w, const float* bias, void* y, int m, int n, int k,
                         int ldy, int epilogue, const NormIn& ni, const NormOut& no, const SplitWorkspace& ws,
                         hipStream_t st, const char** kernel_name) {
    if (linear_mfma_supported(dtype, m, n, k, ldy)) return launch_linear_mfma(x, w, bias, y, m, n, k, ldy, epilogue, ni, no, ws, st, kernel_name);
    if (ni.kind || no.gain) return hipErrorInvalidValue;     // folded normalisations exist on the matrix-core path only
    if (kernel_name) *kernel_name = "k_linear_generic";
    return launch_linear_generic(dtype, x, w, bias, y, m, n, k, ldy, epilogue, st);
}

hipError_t launch_attention(int dtype, const AttnArgs& a, hipStream_t st, const char** kernel_name) {
    if (attention_mfma_supported(dtype, a)) return launch_attention_mfma(a, st, kernel_name);
    if (kernel_name) *kernel_name = "k_attention_generic";
    return launch_attention_generic(dtype, a, a.max_kv, st);
}

}  // namespace sd
