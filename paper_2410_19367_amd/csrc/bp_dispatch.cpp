// Kernel selection: which implementation serves a given GEMM / attention shape.
#include "bp_kernels.h"

namespace bp {

hipError_t launch_gemm(int dtype, const GemmArgs& g, hipStream_t stream) {
    if (dtype == BF16 && gemm_mfma_supported(g)) return launch_gemm_mfma(g, stream);
    return launch_gemm_generic(dtype, g, stream);
}

hipError_t launch_attn_fwd(int dtype, const AttnArgs& a, hipStream_t stream) {
    if (dtype == BF16 && attn_mfma_supported(a)) return launch_attn_fwd_mfma(a, stream);
    return launch_attn_fwd_generic(dtype, a, stream);
}

hipError_t launch_attn_bwd(int dtype, const AttnArgs& a, hipStream_t stream) {
    if (dtype == BF16 && attn_mfma_supported(a)) return launch_attn_bwd_mfma(a, stream);
    return launch_attn_bwd_generic(dtype, a, stream);
}

}  // namespace bp
