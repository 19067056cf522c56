/*
 * bitpipe_stage.h -- C ABI of the MI355X stage-compute library for the BitPipe schedule
 * (arXiv 2410.19367).
 *
 * The unit of work that the paper's bidirectional interleaved schedule orders is the forward or
 * the backward pass of one pipeline stage (a contiguous chunk of transformer layers) on one
 * micro-batch (Section 3.2, Section 3.3; costs t_f and t_b of Appendix B, Eq. 1).  Training is
 * synchronous: weight gradients of all micro-batches of an iteration are accumulated before the
 * flush (Section 1, Section 2).  This library runs that unit of work, and a whole iteration of
 * the V-shaped bidirectional order time-sliced on one GPU, with hand-written gfx950 kernels.
 *
 * One pre-LN layer, row-major activations [tokens, hidden] with token t = b*seq + s:
 *     a   = LN(x; ln1_g, ln1_b)             qkv = a Wqkv + bqkv      (columns [q | k | v],
 *     ctx = softmax(q k^T / sqrt(d) + mask) v                          head-major inside each)
 *     y   = x + ctx Wo + bo
 *     m   = LN(y; ln2_g, ln2_b)             g = GELU_tanh(m W1 + b1)
 *     z   = y + g W2 + b2
 * Weight matrices are row-major [in, out].  LayerNorm uses the biased variance.  The causal mask
 * keeps keys j <= i; the padding mask keeps keys j < len_b (queries are never masked).
 *
 * Conventions
 *   - Every function returns 0 (BP_OK) or a negative bp_status; bp_last_error() returns a
 *     thread-local message for the last failure.  No exception crosses the boundary.
 *   - "dev" pointers are HIP device pointers owned by the caller; "host" pointers are ordinary
 *     host memory.  The library owns weights, gradient accumulators, stashes and workspaces.
 *   - Activation tensors are [microbatch, seq, hidden] in the stage's dtype (BP_BF16: 2-byte
 *     bfloat16; BP_F32: 4-byte float).
 *   - Calls enqueue work on the stage's HIP stream and return without synchronising, except
 *     where stated.  A stage object must not be used from two threads at once.
 */
#ifndef BITPIPE_STAGE_H
#define BITPIPE_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bp_stage bp_stage_t;   /* opaque, library-owned */

enum bp_status {
    BP_OK = 0,
    BP_EINVAL = -1,   /* bad argument (null pointer, index out of range, odd D, ...)      */
    BP_ESHAPE = -2,   /* shape the kernels do not support                                  */
    BP_ESTATE = -3,   /* call order misuse: double forward, backward without forward, ...  */
    BP_EDEP = -4,     /* schedule order fails validation                                    */
    BP_ENOMEM = -5,   /* device or host allocation failed                                   */
    BP_EHIP = -6      /* a HIP runtime call failed                                          */
};

enum bp_dtype { BP_F32 = 0, BP_BF16 = 1 };

/* Parameter tensors of one layer.  Shapes (H = hidden, F = mlp width):
 * LN1_G, LN1_B, LN2_G, LN2_B, BO, B2: [H]; WQKV: [H,3H]; BQKV: [3H]; WO: [H,H];
 * W1: [H,F]; B1: [F]; W2: [F,H]. */
enum bp_tensor_id {
    BP_LN1_G = 0, BP_LN1_B, BP_WQKV, BP_BQKV, BP_WO, BP_BO,
    BP_LN2_G, BP_LN2_B, BP_W1, BP_B1, BP_W2, BP_B2, BP_N_TENSORS
};

typedef struct bp_opts {
    int n_chunks;       /* chunks (stages) held by this object; 0 -> 1                       */
    int mlp;            /* MLP width F; 0 -> 4*hidden (Table 3's 12*L*H^2 parameter count)   */
    int dtype;          /* bp_dtype; storage type of activations and weight matrices          */
    int max_inflight;   /* most (chunk, micro-batch) stashes alive at once; 0 -> 8           */
    float ln_eps;       /* 0 -> 1e-5                                                          */
    void* hip_stream;   /* hipStream_t to enqueue on; NULL -> the default stream             */
    int wgrad_group;    /* weight gradients of this many consecutive backward calls of a chunk
                           and direction are computed together (one pass over the fp32
                           accumulator instead of one per micro-batch); 1: each call computes
                           its own; 2..8; 0 -> min(8, max(1, 16384 / (microbatch*seq))).  A
                           group keeps the stashes of its waiting micro-batches (beyond
                           max_inflight) plus their output gradients until it is complete or
                           until bp_stage_get_grad / bp_run_schedule's merge flushes it.
                           bp_run_schedule uses groups no larger than the number of backward
                           calls a (direction, stage) gets in the iteration.                  */
    int stash_recompute;/* 0: the stash keeps everything the backward reads, 16*T*H elements per
                           layer (x, LN1 out, qkv, ctx, y, LN2 out, u, GELU out); 1: the two
                           LayerNorm outputs and the GELU output are not kept (10*T*H per layer)
                           and are recomputed from x, y, u right before the weight-gradient GEMMs
                           that read them: the activation-memory axis of Table 2               */
    int forward_ahead;  /* 1: bp_stage_forward runs on a stream of the object's own, behind everything
                           the stage's stream holds at the moment of the call, and beside what is
                           enqueued there later: called in the order F(0) F(1) B(0) F(2) B(1) ...
                           (the steady state of the schedules of Section 3, where a device always
                           has the next forward at hand), the forward of one micro-batch overlaps
                           the backward of the one before, filling the CUs that the start and the
                           end of every kernel leave idle.  Results are the same bit for bit.
                           act_out (and act_in, which the forward still reads) belong to the call
                           until the stage's stream has been made to wait for it:
                           bp_stage_wait_forward, the backward of the same micro-batch,
                           bp_stage_get_grad and bp_stage_destroy do that.  0: forwards run on the
                           stage's stream like everything else.  bp_run_schedule ignores it.     */
} bp_opts;

/* Create a stage object holding one chunk of `layers` pre-LN transformer layers in bf16 with
 * fp32 accumulation (the paper's mixed precision, Section 4.1): the compute unit of Section 3.3.
 * causal = 1: GPT-style mask; 0: BERT-style bidirectional attention with optional key padding.
 * Parameters start as LN gamma = 1, everything else 0; gradients start at 0.
 * Requirements: hidden % heads == 0, hidden % 8 == 0, head dim % 8 == 0.
 * Errors: BP_EINVAL, BP_ESHAPE, BP_ENOMEM, BP_EHIP.  *out is set only on success. */
int bp_stage_init(bp_stage_t** out, int layers, int hidden, int heads, int seq,
                  int microbatch, int causal);

/* As bp_stage_init with explicit options (several chunks, fp32 storage, MLP width, stream).
 * opts may be NULL (defaults). */
int bp_stage_init_ex(bp_stage_t** out, int layers, int hidden, int heads, int seq,
                     int microbatch, int causal, const bp_opts* opts);

/* Bytes of activation stash one (chunk, micro-batch) forward keeps until its backward
 * (the M_a of Table 2 for this chunk, statistics included).  0 for a NULL handle. */
size_t bp_stage_stash_bytes(const bp_stage_t* st);

/* Activation memory the object holds right now, in bytes (host bookkeeping, launches nothing): the
 * stashes of forwards whose backward has not run (*live_stash: the activations Table 2 counts in
 * M_a); the stashes kept beyond their backward by weight-gradient groups that are not complete yet
 * (*group_stash) and the output-gradient buffers those groups keep (*group_grads: dz, du, dy, dqkv
 * per layer), both the price of bp_opts.wgrad_group > 1; and the largest sum of the three since the
 * object was created or bp_stage_reset_peak_bytes was called (*peak_total).  Any pointer may be NULL. */
int bp_stage_held_bytes(const bp_stage_t* st, size_t* live_stash, size_t* group_stash, size_t* group_grads,
                        size_t* peak_total);
int bp_stage_reset_peak_bytes(bp_stage_t* st);

/* Synchronise the stream, free everything the object owns.  NULL is accepted. */
int bp_stage_destroy(bp_stage_t* st);

/* Copy one parameter tensor from host fp32 (n elements, must equal the tensor's size) into the
 * library's device copy, rounding weight matrices to the stage dtype (nearest even).
 * Vectors (LN gamma/beta, biases) are kept in fp32.  Synchronous. */
int bp_stage_set_param(bp_stage_t* st, int chunk, int layer, int tensor_id,
                       const float* host_f32, size_t n);

/* Copy one fp32 gradient accumulator to the host (n must equal the tensor's size).
 * Synchronises the stream first.  After bp_run_schedule the two directions are already summed. */
int bp_stage_get_grad(bp_stage_t* st, int chunk, int layer, int tensor_id,
                      float* host_f32, size_t n);

/* Zero all gradient accumulators (the flush between iterations, Section 2).  Launches nothing:
 * the accumulators are marked clear and the first backward of each layer after this call writes
 * its gradient instead of adding it; backward calls already enqueued are not affected. */
int bp_stage_zero_grad(bp_stage_t* st);

/* BERT-style key padding: valid lengths (host int32 [microbatch], each in 1..seq) used by the
 * forward and backward of micro-batch `mb` from now on; lens = NULL clears them (full length).
 * BP_ESTATE on a causal stage or while `mb` has a live stash. */
int bp_stage_set_seqlens(bp_stage_t* st, int mb, const int32_t* lens_host);

/* Forward of chunk `chunk` on micro-batch `mb` (the box "F" of the paper's schedule figures):
 * act_in (dev, [B,S,H]) -> act_out (dev, [B,S,H]); what the backward needs is stashed under
 * (chunk, mb).  act_out may be the act_in of the next stage's forward (that hand-off is the
 * paper's P2P message or, at the V turn, its local copy -- Section 3.2); act_in and act_out must
 * not overlap.  BP_ESTATE: (chunk, mb) already stashed, or max_inflight stashes alive. */
int bp_stage_forward(bp_stage_t* st, int chunk, int mb, const void* act_in, void* act_out);

/* Backward of chunk `chunk` on micro-batch `mb` (the box "B"): grad_out (dev, [B,S,H], gradient
 * w.r.t. the chunk's output) -> grad_in (dev, [B,S,H], w.r.t. its input); every parameter
 * gradient of the chunk is accumulated in fp32 (+=) and the stash of (chunk, mb) is released.
 * grad_in may alias grad_out.  BP_ESTATE: no stashed forward for (chunk, mb). */
int bp_stage_backward(bp_stage_t* st, int chunk, int mb, const void* grad_out, void* grad_in);

/* As bp_stage_backward, accumulating into the gradient buffer of pipeline direction `direction`
 * (0 down, 1 up): the two replicas of a stage that Section 3.4's all-reduce synchronises. */
int bp_stage_backward_dir(bp_stage_t* st, int chunk, int mb, const void* grad_out,
                          void* grad_in, int direction);

/* Add the direction-1 accumulators into the direction-0 ones and clear direction 1: the sum that
 * stands in, on one device, for the all-reduce between the two replicas of a stage (Section 3.4).
 * bp_run_schedule does this at the end of an iteration; a caller that drives the two pipelines
 * itself with bp_stage_backward_dir calls it before bp_stage_get_grad, which reads direction 0.
 * Completes the weight-gradient groups still open first.  Asynchronous (enqueued on the object's
 * streams; bp_stage_get_grad synchronises).  Calling it twice in a row adds nothing the second time. */
int bp_stage_merge_directions(bp_stage_t* st);

/* With bp_opts.forward_ahead: make the stage's stream wait for every forward enqueued so far, so
 * that work enqueued on it afterwards (the caller's consumer of act_out, a copy to the next stage)
 * sees their outputs.  Asynchronous; without forward_ahead it does nothing.  Errors: BP_EINVAL, BP_EHIP. */
int bp_stage_wait_forward(bp_stage_t* st);

/* One operation of a schedule: forward or backward of global stage `stage` (= chunk index) on
 * micro-batch `mb`, in pipeline `dir`, placed on virtual device `vdev`. */
typedef struct bp_op {
    int8_t kind;      /* 0 forward, 1 backward */
    int8_t dir;       /* 0 down pipeline, 1 up pipeline */
    int16_t vdev;     /* virtual device 0..D-1 */
    int32_t stage;    /* 0..2D-1 */
    int32_t mb;       /* 0..N-1 */
} bp_op;

/* BP_SCHED_V_CONCAT: basic units concatenated (Section 3.5).  BP_SCHED_V_EARLY_FWD: early
 * forwarding (Appendix B): forwards of later micro-batches run ahead of time, removing the bubbles
 * between units at the price of up to 3D-3 instead of 2D chunk stashes per device. */
enum bp_schedule_variant { BP_SCHED_V_CONCAT = 0, BP_SCHED_V_EARLY_FWD = 1 };

/* Pure CPU.  Stage -> virtual device of the V-shaped map (Section 3.2, Section 3.3):
 * down: 0..D-1 then D-1..0; up: the mirror image.  Returns -1 on bad arguments. */
int bp_schedule_vmap(int dir, int stage, int D);

/* Pure CPU.  Write the serial order of one BitPipe iteration with D virtual devices, 2D stages
 * and N micro-batches (N a multiple of D, D even; Section 3.3 basic unit, Section 3.5
 * concatenation) into out[0..cap); *n_out = 4*D*N ops.  The order is a list schedule under the
 * paper's cost model (chunk forward 1, backward 2), serialised by (start time, device).  Each
 * pipeline runs its micro-batches by the 1F1B-Int rule (Section 3.3): a free device takes the ready
 * backward of the micro-batch that entered its own pipeline first (not starting one that would delay
 * a more urgent backward due in the next slot), else the ready forward of the deepest stage.
 * What the orders reach when replayed by bp_schedule_simulate:
 *   CONCAT, N = D (the basic unit): the closed forms of Section 3.3 / Table 2 -- makespan
 *     2(3N+D-2) chunk slots, bubble ratio (D-2)/(3N+D-2), at most D M_a -- for every even D tested
 *     (4, 6, 8, 10, 12, 16);
 *   CONCAT, N = K*D: valid, better than K units back to back, within a few per cent of the closed
 *     form but not equal to it (e.g. 53 against 52 slots at D = 4, N = 8);
 *   EARLY_FWD: (D-2)/(4N+D-2) and peak (3D-3)/2 M_a at D = 4, N = 2D..6D and at D = 6, N = 12;
 *     valid but above the closed form elsewhere.
 * BP_EINVAL for odd D, N % D != 0, cap too small or an unknown variant. */
int bp_schedule_generate(int D, int N, int variant, bp_op* out, int cap, int* n_out);

/* Pure CPU.  BP_OK iff the order holds exactly one forward and one backward per (stage, mb),
 * every op comes after the ops it depends on, vdev matches the V map and a micro-batch keeps
 * one direction; else BP_EDEP (bp_last_error names the first violation). */
int bp_schedule_validate(const bp_op* order, int n_ops, int D, int N);

/* Pure CPU.  Simulate `order` under the cost model (forward cost_f, backward cost_b per chunk)
 * with each op starting as soon as its device and its inputs are free, keeping the list's
 * per-device order.  Outputs (each may be NULL): makespan, idle[D] per device, peak_stash[D]. */
int bp_schedule_simulate(const bp_op* order, int n_ops, int D, int N, int cost_f, int cost_b,
                         int* makespan, int* idle, int* peak_stash);

/* Run a whole iteration on one GPU (Section 3.3 / 3.5 order, all virtual devices time-sliced).
 * The object must hold n_chunks == 2*D chunks.  order is validated first (BP_EDEP, nothing is
 * launched); gradients are zeroed; ops run in list order, the output of stage s feeding stage
 * s+1 (the emulated P2P / local copy); after the last stage's forward of micro-batch m the loss
 *     L_m = 1/(N*B*S) * sum_{b,s} 0.5 * || z_m[b,s,:] - targets[m,b,s,:] ||^2
 * and its gradient seed the backward; backward ops accumulate into their direction's gradient
 * buffer and at the end the two are summed (the all-reduce of Section 3.4 on one device).
 * inputs, targets: dev [N,B,S,H] in the stage dtype.  loss_out (host, may be NULL) receives
 * sum_m L_m.  Synchronises before returning. */
int bp_run_schedule(bp_stage_t* st, const bp_op* order, int n_ops, int D,
                    const void* inputs_dev, const void* targets_dev, float* loss_out);

/* ---- other stage placements (Appendix A; the "w/o V" ablation of Section 4.4).
 * v: chunks per device and pipeline, so a pipeline has v*D stages (the default V shape is v = 2;
 * v = 1 is one chunk per device and direction).  looping = 0: the walk over the devices turns
 * round at both ends (0..D-1, D-1..0, 0..D-1, ...), every turn being a local copy; looping = 1:
 * the placement of the plain interleaved schedule, which restarts at device 0 after each lap and
 * has no local copies.  A NULL layout means {2, 0}.  The *_ex calls below are the calls above for
 * an arbitrary layout: stages run from 0 to v*D-1, an order holds 2*v*D*N ops, the stage object
 * must hold v*D chunks.  Stash caps of the list scheduler scale with v (a stage-activation M_a is
 * v chunk stashes).  The closed forms of the paper are pinned for {2, 0} only. */
typedef struct bp_layout {
    int v;
    int looping;
} bp_layout;

int bp_schedule_vmap_ex(const bp_layout* layout, int dir, int stage, int D);
int bp_schedule_generate_ex(const bp_layout* layout, int D, int N, int variant, bp_op* out, int cap,
                            int* n_out);
int bp_schedule_validate_ex(const bp_layout* layout, const bp_op* order, int n_ops, int D, int N);
int bp_schedule_simulate_ex(const bp_layout* layout, const bp_op* order, int n_ops, int D, int N,
                            int cost_f, int cost_b, int* makespan, int* idle, int* peak_stash);
int bp_run_schedule_ex(bp_stage_t* st, const bp_layout* layout, const bp_op* order, int n_ops, int D,
                       const void* inputs, const void* targets, float* loss_out);

/* Pure CPU.  Messages of one iteration under a layout: every forward hands its output to the next
 * stage and every backward its input gradient to the previous one.  *p2p counts the hand-overs
 * between different devices (each a message of 2*B*S*H bytes, Appendix C), *local those that stay
 * on a device.  For the zig-zag map: p2p = 2*N*v*(D-1), local = 2*N*(v-1); looping: p2p =
 * 2*N*(v*D-1), local = 0.  Either output pointer may be NULL.  Errors as bp_schedule_validate. */
int bp_schedule_hops(const bp_layout* layout, const bp_op* order, int n_ops, int D, int N,
                     long* p2p, long* local);

/* ---- per-kernel timing (HIP events recorded on the stage's stream around every launch) ---- */

enum bp_kernel_id {
    BP_K_GEMM = 0,        /* all linear-layer GEMMs: forward, dgrad, wgrad          */
    BP_K_ATTN_FWD,
    BP_K_ATTN_BWD,
    BP_K_LN_FWD,
    BP_K_LN_BWD,
    BP_K_GELU_FWD,
    BP_K_GELU_BWD,
    BP_K_COLSUM,          /* bias / LN parameter gradient column reductions         */
    BP_K_OTHER,           /* copies, casts, loss, gradient merge                    */
    BP_N_KERNEL_IDS
};

/* Turn event timing on (1) or off (0) and clear the counters.  While on, every launch is
 * bracketed by two events on the stage's stream; off is the default and costs nothing. */
int bp_prof_enable(bp_stage_t* st, int on);

/* Synchronise and read the totals of one kernel class since bp_prof_enable(st, 1):
 * milliseconds between the events, number of launches, algorithmic flops and algorithmic bytes
 * (what the class had to compute / move by the layer definition, not what it actually did). */
int bp_prof_get(bp_stage_t* st, int kernel_id, double* total_ms, long long* launches,
                double* flops, double* bytes);

/* Per-shape totals of the GEMM class since bp_prof_enable(st, 1).  bp_prof_gemm_shapes returns the
 * number of distinct GEMM shapes launched (>= 0, or a negative bp_status); bp_prof_gemm_get reads
 * entry `index`: dims[7] = {M, N, K of one contraction segment, a_t, b_t, segments, epilogue (0 none,
 * 1 bias+GELU forward, 2 GELU backward + bias-gradient partials)} in the sense of bp_op_gemm /
 * bp_op_wgrad_group, the milliseconds between the launches' events (a split-K GEMM includes its
 * reduction kernel) and the launch count.  Both synchronise.  Any output pointer may be NULL. */
int bp_prof_gemm_shapes(bp_stage_t* st);
int bp_prof_gemm_get(bp_stage_t* st, int index, int* dims, double* total_ms, long long* launches);

/* ---- single operations on caller-owned device buffers (tests and kernel benchmarks) ------ */

/* C = op(A) * op(B) (+ bias) (+ residual), or C += op(A) * op(B) when accumulate != 0.
 * dtype: storage type of A, B, residual and (when accumulate == 0) C; with accumulate != 0, C is
 * fp32.  op(A) is [M,K]: a_t == 0 -> A[m*lda + k]; a_t != 0 -> A[k*lda + m].  op(B) is [K,N]:
 * b_t == 0 -> B[k*ldb + n]; b_t != 0 -> B[n*ldb + k].  bias: fp32 [N] or NULL.  residual: [M,N]
 * leading dimension ldc, or NULL.  These are the three shapes of a linear layer: forward
 * (a_t=0,b_t=0), dgrad (0,1) and wgrad (1,0, accumulate).  stream: hipStream_t or NULL. */
int bp_op_gemm(int dtype, int a_t, int b_t, int M, int N, int K,
               const void* A, int lda, const void* B, int ldb, void* C, int ldc,
               const float* bias, const void* residual, int accumulate, void* stream);

/* Weight gradient of a linear map over a group of n micro-batches (1 <= n <= 8) in one pass over
 * the fp32 accumulator: dW (+)= sum_i X[i]^T dY[i], the synchronous gradient accumulation of
 * Section 2 with the sum over micro-batches moved inside the contraction.
 * X: host array of n device pointers, each [T, M] row-major in `dtype`; dY: likewise [T, N];
 * dW: dev fp32 [M, N].  overwrite != 0: dW = instead of dW +=.
 * workspace: optional dev fp32 scratch of workspace_elems floats (NULL / 0: none).  With it, the
 * output tiles that do not fill the chip (all of them for a small dW, else those of the last,
 * partly filled round) are cut into up to 4 slices of a long token axis that run on different
 * CUs; their partial sums go through the workspace (4*M*N floats always suffice) and are added
 * in a fixed order.  Asynchronous on `stream`. */
int bp_op_wgrad_group(int dtype, int M, int N, int T, int n, const void* const* X,
                      const void* const* dY, float* dW, int overwrite, float* workspace,
                      size_t workspace_elems, void* stream);

/* out = LN(x) over rows of [T,H]; writes mean and rstd (fp32 [T]). */
int bp_op_layernorm_fwd(int dtype, int T, int H, const void* x, const float* gamma,
                        const float* beta, float eps, void* out, float* mean, float* rstd,
                        void* stream);

/* dx = residual_grad + LNbwd(dout) (residual_grad may be NULL); dgamma, dbeta (fp32 [H]) are
 * accumulated (+=).  workspace: dev fp32, at least bp_op_colsum_workspace(T, H) * 2 floats. */
int bp_op_layernorm_bwd(int dtype, int T, int H, const void* dout, const void* x,
                        const float* mean, const float* rstd, const float* gamma,
                        const void* residual_grad, void* dx, float* dgamma, float* dbeta,
                        float* workspace, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): bp_op_layernorm_bwd without the workspace argument.  The
 * column-reduction partials go to a device array that is part of the library image:
 * bp_static_scratch_floats() floats (8 MiB) per GPU, held from the library's first use of that GPU
 * until the process ends.  Needs (T + 31) / 32 * 2 * H floats; larger problems return BP_ESHAPE
 * (use bp_op_layernorm_bwd with a workspace).  The call makes no hipMalloc / hipFree and calls no
 * allocating routine; it looks the array's device address up once per device (the device current
 * at the call).  All calls on one GPU share the array: calls that overlap on one GPU (two streams,
 * two threads) race, calls on one stream are ordered.  Nothing in it needs clearing between calls.
 * Arguments, results and errors otherwise as bp_op_layernorm_bwd. */
size_t bp_static_scratch_floats(void);
int bp_op_layernorm_bwd_static(int dtype, int T, int H, const void* dout, const void* x,
                               const float* mean, const float* rstd, const float* gamma,
                               const void* residual_grad, void* dx, float* dgamma, float* dbeta,
                               void* stream);

/* g = GELU_tanh(u + bias) over [T,F]. */
int bp_op_bias_gelu_fwd(int dtype, int T, int F, const void* u, const float* bias, void* g,
                        void* stream);

/* du = dg * GELU'(u + bias); dbias (fp32 [F]) += column sums of du.  workspace as above. */
int bp_op_bias_gelu_bwd(int dtype, int T, int F, const void* dg, const void* u,
                        const float* bias, void* du, float* dbias, float* workspace,
                        void* stream);

/* Number of fp32 elements of workspace one column reduction over [T,N] needs. */
size_t bp_op_colsum_workspace(int T, int N);

/* Fused attention forward on a packed qkv tensor [B*S, 3H] (columns [q|k|v], head-major):
 * ctx [B*S, H], lse fp32 [B, heads, S] (log-sum-exp of the scaled, masked scores).
 * lens: dev int32 [B] or NULL. */
int bp_op_attention_fwd(int dtype, int B, int S, int heads, int head_dim, int causal,
                        const int32_t* lens_dev, const void* qkv, void* ctx, float* lse,
                        void* stream);

/* Fused attention backward: dqkv [B*S, 3H] from dctx, the forward's qkv, ctx and lse.
 * delta: dev fp32 workspace [B, heads, S]. */
int bp_op_attention_bwd(int dtype, int B, int S, int heads, int head_dim, int causal,
                        const int32_t* lens_dev, const void* qkv, const void* ctx,
                        const float* lse, const void* dctx, void* dqkv, float* delta,
                        void* stream);

/* Message of the last failure on this thread ("" if none). */
const char* bp_last_error(void);

/* Library version string. */
const char* bp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BITPIPE_STAGE_H */
