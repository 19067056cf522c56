// C ABI of the single operations (caller-owned device buffers): argument checks, then the same
// launchers the stage uses.
#include "bp_host.h"

using bp::fail;

#define BP_OP_LAUNCH(expr)                                                              \
    do {                                                                                \
        hipError_t e_ = (expr);                                                         \
        if (e_ != hipSuccess) return fail(BP_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
        return BP_OK;                                                                   \
    } while (0)

static int check_dtype(int dtype) {
    if (dtype != BP_F32 && dtype != BP_BF16) return fail(BP_EINVAL, "unknown dtype %d", dtype);
    return BP_OK;
}

extern "C" {

int bp_op_gemm(int dtype, int a_t, int b_t, int M, int N, int K, const void* A, int lda,
               const void* B, int ldb, void* C, int ldc, const float* bias, const void* residual,
               int accumulate, void* stream) {
    if (check_dtype(dtype)) return BP_EINVAL;
    if (!A || !B || !C) return fail(BP_EINVAL, "null matrix pointer");
    if (M <= 0 || N <= 0 || K <= 0) return fail(BP_EINVAL, "M, N, K must be positive");
    if (lda < (a_t ? M : K) || ldb < (b_t ? K : N) || ldc < N)
        return fail(BP_EINVAL, "leading dimension smaller than the row length");
    if (accumulate && (bias || residual))
        return fail(BP_EINVAL, "accumulate excludes bias and residual");
    bp::GemmArgs g;
    g.A = A; g.B = B; g.C = C; g.bias = bias; g.residual = residual;
    g.M = M; g.N = N; g.K = K; g.lda = lda; g.ldb = ldb; g.ldc = ldc;
    g.a_t = a_t != 0; g.b_t = b_t != 0; g.accumulate = accumulate != 0;
    BP_OP_LAUNCH(bp::launch_gemm(dtype, g, (hipStream_t)stream));
}

int bp_op_wgrad_group(int dtype, int M, int N, int T, int n, const void* const* X, const void* const* dY,
                      float* dW, int overwrite, float* workspace, size_t workspace_elems, void* stream) {
    if (check_dtype(dtype)) return BP_EINVAL;
    if (!X || !dY || !dW) return fail(BP_EINVAL, "null pointer");
    if (M <= 0 || N <= 0 || T <= 0) return fail(BP_EINVAL, "M, N, T must be positive");
    if (n < 1 || n > bp::kMaxGemmSegments)
        return fail(BP_EINVAL, "n = %d outside 1..%d", n, bp::kMaxGemmSegments);
    for (int i = 0; i < n; ++i)
        if (!X[i] || !dY[i]) return fail(BP_EINVAL, "null operand %d", i);
    bp::GemmArgs g;
    g.A = X[0]; g.B = dY[0]; g.C = dW; g.bias = nullptr; g.residual = nullptr;
    g.M = M; g.N = N; g.K = T; g.lda = M; g.ldb = N; g.ldc = N;
    g.a_t = 1; g.b_t = 0; g.accumulate = overwrite ? 2 : 1;
    g.nseg = n;
    for (int i = 1; i < n; ++i) { g.A_more[i - 1] = X[i]; g.B_more[i - 1] = dY[i]; }
    if (workspace && workspace_elems) { g.split_ws = workspace; g.split_ws_elems = workspace_elems; }
    BP_OP_LAUNCH(bp::launch_gemm(dtype, g, (hipStream_t)stream));
}

int bp_op_layernorm_fwd(int dtype, int T, int H, const void* x, const float* gamma, const float* beta,
                        float eps, void* out, float* mean, float* rstd, void* stream) {
    if (check_dtype(dtype)) return BP_EINVAL;
    if (!x || !gamma || !beta || !out || !mean || !rstd) return fail(BP_EINVAL, "null pointer");
    if (T <= 0 || H <= 0) return fail(BP_EINVAL, "T and H must be positive");
    if (H % 8 || H > 8192) return fail(BP_ESHAPE, "H = %d must be a multiple of 8 and at most 8192", H);
    BP_OP_LAUNCH(bp::launch_ln_fwd(dtype, T, H, x, gamma, beta, eps, out, mean, rstd, nullptr,
                                   (hipStream_t)stream));
}

int bp_op_layernorm_bwd(int dtype, int T, int H, const void* dout, const void* x, const float* mean,
                        const float* rstd, const float* gamma, const void* residual_grad, void* dx,
                        float* dgamma, float* dbeta, float* workspace, void* stream) {
    if (check_dtype(dtype)) return BP_EINVAL;
    if (!dout || !x || !mean || !rstd || !gamma || !dx || !dgamma || !dbeta || !workspace)
        return fail(BP_EINVAL, "null pointer");
    if (T <= 0 || H <= 0) return fail(BP_EINVAL, "T and H must be positive");
    if (H % 8 || H > 8192) return fail(BP_ESHAPE, "H = %d must be a multiple of 8 and at most 8192", H);
    hipError_t e = bp::launch_colsum(dtype, T, H, dout, x, mean, rstd, dbeta, dgamma, workspace,
                                     (hipStream_t)stream);
    if (e != hipSuccess) return fail(BP_EHIP, "column reduction: %s", hipGetErrorString(e));
    BP_OP_LAUNCH(bp::launch_ln_bwd_rows(dtype, T, H, dout, x, mean, rstd, gamma, residual_grad, dx,
                                        (hipStream_t)stream));
}

int bp_op_bias_gelu_fwd(int dtype, int T, int F, const void* u, const float* bias, void* g, void* stream) {
    if (check_dtype(dtype)) return BP_EINVAL;
    if (!u || !bias || !g) return fail(BP_EINVAL, "null pointer");
    if (T <= 0 || F <= 0) return fail(BP_EINVAL, "T and F must be positive");
    if (F % 8) return fail(BP_ESHAPE, "F = %d must be a multiple of 8", F);
    BP_OP_LAUNCH(bp::launch_gelu_fwd(dtype, T, F, u, bias, g, (hipStream_t)stream));
}

int bp_op_bias_gelu_bwd(int dtype, int T, int F, const void* dg, const void* u, const float* bias,
                        void* du, float* dbias, float* workspace, void* stream) {
    if (check_dtype(dtype)) return BP_EINVAL;
    if (!dg || !u || !bias || !du || !dbias || !workspace) return fail(BP_EINVAL, "null pointer");
    if (T <= 0 || F <= 0) return fail(BP_EINVAL, "T and F must be positive");
    if (F % 8) return fail(BP_ESHAPE, "F = %d must be a multiple of 8", F);
    BP_OP_LAUNCH(bp::launch_gelu_bwd(dtype, T, F, dg, u, bias, du, dbias, workspace, (hipStream_t)stream));
}

size_t bp_op_colsum_workspace(int T, int N) {
    if (T <= 0 || N <= 0) return 0;
    return bp::colsum_chunks(T) * (size_t)N;
}

static int check_attn(int dtype, int B, int S, int heads, int head_dim) {
    if (check_dtype(dtype)) return BP_EINVAL;
    if (B <= 0 || S <= 0 || heads <= 0 || head_dim <= 0) return fail(BP_EINVAL, "B, S, heads, head_dim must be positive");
    if (head_dim % 8) return fail(BP_ESHAPE, "head_dim = %d must be a multiple of 8", head_dim);
    if ((size_t)S * sizeof(float) * 2 > 56000) return fail(BP_ESHAPE, "S = %d too long", S);
    return BP_OK;
}

int bp_op_attention_fwd(int dtype, int B, int S, int heads, int head_dim, int causal,
                        const int32_t* lens, const void* qkv, void* ctx, float* lse, void* stream) {
    int rc = check_attn(dtype, B, S, heads, head_dim);
    if (rc) return rc;
    if (!qkv || !ctx || !lse) return fail(BP_EINVAL, "null pointer");
    bp::AttnArgs a{B, S, heads, head_dim, causal != 0, causal ? nullptr : lens, qkv, ctx, lse,
                   nullptr, nullptr, nullptr};
    BP_OP_LAUNCH(bp::launch_attn_fwd(dtype, a, (hipStream_t)stream));
}

int bp_op_attention_bwd(int dtype, int B, int S, int heads, int head_dim, int causal,
                        const int32_t* lens, const void* qkv, const void* ctx, const float* lse,
                        const void* dctx, void* dqkv, float* delta, void* stream) {
    int rc = check_attn(dtype, B, S, heads, head_dim);
    if (rc) return rc;
    if (!qkv || !ctx || !lse || !dctx || !dqkv || !delta) return fail(BP_EINVAL, "null pointer");
    bp::AttnArgs a{B, S, heads, head_dim, causal != 0, causal ? nullptr : lens, qkv, (void*)ctx,
                   (float*)lse, dctx, dqkv, delta};
    BP_OP_LAUNCH(bp::launch_attn_bwd(dtype, a, (hipStream_t)stream));
}

}  // extern "C"
