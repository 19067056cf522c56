// Kernel selection: which implementation serves a given GEMM / attention shape.
#include "bp_kernels.h"

namespace bp {

// one launch per contraction segment, for kernels that take a single operand pair
hipError_t launch_gemm_per_segment(const GemmArgs& g, hipStream_t stream,
                                   hipError_t (*one)(const GemmArgs&, hipStream_t)) {
    GemmArgs h = g;
    h.nseg = 1;
    for (int sgm = 0; sgm < g.nseg; ++sgm) {
        if (sgm > 0) {
            h.A = g.A_more[sgm - 1];
            h.B = g.B_more[sgm - 1];
            h.accumulate = 1;
        }
        hipError_t e = one(h, stream);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_gemm(int dtype, const GemmArgs& g, hipStream_t stream) {
    if (g.nseg < 1 || g.nseg > kMaxGemmSegments || (g.nseg > 1 && !g.accumulate)) return hipErrorInvalidValue;
    if (g.epi != EPI_NONE && !gemm_can_fuse_epilogue(dtype, g)) return hipErrorInvalidValue;
    if (dtype == BF16 && gemm_mfma_supported(g)) return launch_gemm_mfma(g, stream);
    if (g.nseg == 1) return launch_gemm_generic(dtype, g, stream);
    if (dtype == BF16)
        return launch_gemm_per_segment(g, stream, [](const GemmArgs& h, hipStream_t s) {
            return launch_gemm_generic(BF16, h, s);
        });
    return launch_gemm_per_segment(g, stream, [](const GemmArgs& h, hipStream_t s) {
        return launch_gemm_generic(F32, h, s);
    });
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
