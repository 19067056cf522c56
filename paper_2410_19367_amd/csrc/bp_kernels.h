// Internal launch interface between the host-side stage logic and the gfx950 kernels.
// Every function enqueues on `stream` and returns the launch status; none synchronises.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace bp {

enum DType { F32 = 0, BF16 = 1 };

inline size_t dtype_size(int dt) { return dt == BF16 ? 2 : 4; }

constexpr int kMaxGemmSegments = 8;

// C = op(A) op(B) (+bias) (+residual)  or  C(fp32) += op(A) op(B).
//   op(A)[m,k] = a_t ? A[k*lda + m] : A[m*lda + k]
//   op(B)[k,n] = b_t ? B[n*ldb + k] : B[k*ldb + n]
struct GemmArgs {
    const void* A; const void* B; void* C;
    const float* bias;       // [N] or null
    const void* residual;    // [M,N] ld = ldc, storage dtype, or null
    int M, N, K;
    int lda, ldb, ldc;
    int a_t, b_t;
    int accumulate;          // 1: C is fp32 and receives +=;  2: C is fp32 and is overwritten (= instead of +=)
    // optional split-K workspace (fp32, split_ws_elems floats).  When given, the output tiles that
    // would leave much of the chip idle (all of them when they are few, else those of a partly
    // filled last round) may have K cut into up to 4 slices computed by different blocks, each
    // writing an fp32 partial of its tile there; a second kernel adds the partials in a fixed
    // order and applies the epilogue.  splits * tiles * tile size floats are needed; 4 * M * N
    // always suffice.  Null: never split.
    float* split_ws = nullptr;
    size_t split_ws_elems = 0;
    // Optional further contraction segments: the product runs over nseg operand pairs
    // (A, B), (A_more[0], B_more[0]), ... of K each, all with the same lda / ldb, as if the pairs
    // were concatenated along the contraction index (weight gradient of several micro-batches in
    // one pass over the fp32 accumulator).
    int nseg = 1;
    const void* A_more[kMaxGemmSegments - 1] = {};
    const void* B_more[kMaxGemmSegments - 1] = {};
    // Optional fused GELU epilogue (only with accumulate == 0 and no residual; honoured when
    // gemm_can_fuse_epilogue() says so, callers run the separate kernels otherwise):
    //   EPI_GELU_FWD : C = product (no bias), C2 = gelu(product + bias)
    //   EPI_GELU_BWD : C = product * gelu'(U + bias), and colpart[r][n] = sum of C over rows
    //                  32r .. 32r+31 (fp32, [M/32][N]), the partials of the bias gradient
    int epi = 0;
    void* C2 = nullptr;          // [M,N] ld = ldc
    const void* U = nullptr;     // [M,N] ld = ldc
    float* colpart = nullptr;
};
enum { EPI_NONE = 0, EPI_GELU_FWD = 1, EPI_GELU_BWD = 2 };
bool gemm_can_fuse_epilogue(int dtype, const GemmArgs& g);

// picks the MFMA kernel when the shape allows it, else the generic one
hipError_t launch_gemm(int dtype, const GemmArgs& g, hipStream_t stream);
hipError_t launch_gemm_generic(int dtype, const GemmArgs& g, hipStream_t stream);
bool gemm_mfma_supported(const GemmArgs& g);                       // bf16 only
hipError_t launch_gemm_mfma(const GemmArgs& g, hipStream_t stream);
hipError_t launch_gemm_per_segment(const GemmArgs& g, hipStream_t stream,
                                   hipError_t (*one)(const GemmArgs&, hipStream_t));

// rows kept per partial of a column reduction
constexpr int kColsumRows = 32;
inline size_t colsum_chunks(int T) { return (size_t)((T + kColsumRows - 1) / kColsumRows); }

hipError_t launch_ln_fwd(int dtype, int T, int H, const void* x, const float* gamma,
                         const float* beta, float eps, void* out, float* mean, float* rstd,
                         void* xcopy, hipStream_t stream);

// dx = res + LNbwd(dout) row by row (res may be null)
hipError_t launch_ln_bwd_rows(int dtype, int T, int H, const void* dout, const void* x,
                              const float* mean, const float* rstd, const float* gamma,
                              const void* res, void* dx, hipStream_t stream);

// Column reductions over [T,N] into fp32 accumulators (+=):
//   out_a[c]  += sum_t A[t,c]
//   out_ax[c] += sum_t A[t,c] * (X[t,c]-mean[t])*rstd[t]     (only when X != null)
// ws: colsum_chunks(T) * N * (X ? 2 : 1) floats.
// A batch of column reductions over tensors with the same number of rows.  A job with A == null
// only folds partials that another kernel already left in `part` (chunk-major [chunks][N]).
struct ColsumJob {
    const void* A;        // [T,N] storage dtype, or null
    const void* X;        // [T,N] or null; with X: out_ax += sum_t A * (X - mean) * rstd
    const float* mean;
    const float* rstd;
    int N;
    float* out_a;         // += sum_t A
    float* out_ax;        // or null
    float* part;          // colsum_chunks(T) * N * (out_ax ? 2 : 1) floats
};
constexpr int kMaxColsumJobs = 8;
struct ColsumBatch {
    ColsumJob jobs[kMaxColsumJobs];
    int n;
    int overwrite = 0;       // 1: outputs receive = instead of +=
    // filled by launch_colsum_batch: first column-block id of each job in the flattened grid of the
    // partial kernel (jobs without a tensor own no blocks)
    int first_block[kMaxColsumJobs + 1] = {};
};
hipError_t launch_colsum_batch(int dtype, int T, const ColsumBatch& batch, hipStream_t stream);

hipError_t launch_colsum(int dtype, int T, int N, const void* A, const void* X,
                         const float* mean, const float* rstd, float* out_a, float* out_ax,
                         float* ws, hipStream_t stream);

hipError_t launch_gelu_fwd(int dtype, int T, int F, const void* u, const float* bias, void* g,
                           hipStream_t stream);

// du = dg * gelu'(u + bias); dbias += colsum(du).  ws: colsum_chunks(T) * F floats.
hipError_t launch_gelu_bwd(int dtype, int T, int F, const void* dg, const void* u,
                           const float* bias, void* du, float* dbias, float* ws,
                           hipStream_t stream);

struct AttnArgs {
    int B, S, heads, d, causal;
    const int32_t* lens;     // dev [B] or null
    const void* qkv;         // [B*S, 3*heads*d]
    void* ctx;               // fwd: out; bwd: in  [B*S, heads*d]
    float* lse;              // [B, heads, S]
    const void* dctx;        // bwd
    void* dqkv;              // bwd out
    float* delta;            // bwd workspace [B, heads, S]
};
hipError_t launch_attn_fwd(int dtype, const AttnArgs& a, hipStream_t stream);
hipError_t launch_attn_bwd(int dtype, const AttnArgs& a, hipStream_t stream);
bool attn_mfma_supported(const AttnArgs& a);                       // bf16, head dim 64/128, S % 64 == 0
hipError_t launch_attn_fwd_mfma(const AttnArgs& a, hipStream_t stream);
hipError_t launch_attn_bwd_mfma(const AttnArgs& a, hipStream_t stream);
hipError_t launch_attn_fwd_generic(int dtype, const AttnArgs& a, hipStream_t stream);
hipError_t launch_attn_bwd_generic(int dtype, const AttnArgs& a, hipStream_t stream);

// grad = (z - target) * scale in the storage dtype; loss_out[0] = 0.5 * scale * sum (z-target)^2.
// ws: at least 1024 floats.
hipError_t launch_loss(int dtype, size_t n, const void* z, const void* target, float scale,
                       void* grad, float* loss_out, float* ws, hipStream_t stream);

hipError_t launch_fill_f32(float* p, size_t n, float v, hipStream_t stream);
hipError_t launch_add_f32(float* dst, const float* src, size_t n, hipStream_t stream);   // dst += src
// host fp32 staging (already on device as fp32) -> storage dtype
// dst[cols][rows] = src[rows][cols]^T, storage dtype
hipError_t launch_transpose(int dtype, int rows, int cols, const void* src, void* dst, hipStream_t stream);
hipError_t launch_cast_from_f32(int dtype, const float* src, void* dst, size_t n, hipStream_t stream);

}  // namespace bp
