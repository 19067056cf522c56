// Host-side types of the stage library (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>

#include <map>
#include <new>
#include <string>
#include <vector>

#include "../../include/bitpipe_stage.h"
#include "bp_kernels.h"

namespace bp {

int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
const char* last_error();

struct Stage;

// Stage placement of a pipeline: v chunks per device, zig-zag (the V shape for v = 2) or looping.
struct Layout {
    int v = 2;
    bool looping = false;
};

// Optional event timing of every launch, grouped by kernel class.
struct Prof {
    struct Pending { int kid; hipEvent_t start, stop; int shape; };
    // GEMM launches are also totalled per shape: {M, N, K per segment, a_t, b_t, segments, epilogue}
    struct ShapeStat { int dims[7]; double ms; long long launches; };
    std::vector<ShapeStat> shapes;
    int next_shape = -1;       // shape slot of the launch that begin() is about to record
    void tag_gemm(int M, int N, int K, int a_t, int b_t, int nseg, int epi);
    bool on = false;
    std::vector<Pending> pending;
    std::vector<hipEvent_t> free_events;
    double ms_total[BP_N_KERNEL_IDS] = {};
    double flops_total[BP_N_KERNEL_IDS] = {};
    double bytes_total[BP_N_KERNEL_IDS] = {};
    long long launches[BP_N_KERNEL_IDS] = {};
    void begin(Stage* st, int kid, double flops, double bytes);
    void end(Stage* st);
    void collect();
    void reset();
    ~Prof();
};

struct StashSlot {
    void* buf = nullptr;   // L * s_layer_bytes, allocated on first use and kept
    bool live = false;
    int chunk = -1, mb = -1;
    hipEvent_t side_done = nullptr;   // last side-stream reader of this slot (null: none pending)
    bool side_pending = false;
    hipEvent_t fwd_done = nullptr;    // end of the forward that filled this slot, on the forward stream
    bool fwd_pending = false;
    bool held = false;     // backward done, but the weight gradients of its group are still to come
};

// A micro-batch whose backward has run but whose weight-gradient GEMMs wait for the rest of its
// group: its stash slot stays held and `buf` keeps, per layer, the gradients w.r.t. the outputs
// of the four linear maps (dz, du, dy, dqkv).
struct PendingMb { int slot; void* buf; };
struct PendGroup { std::vector<PendingMb> items; };

// Everything one stream pair needs to run forwards and backwards on its own: the streams, the
// events that order the two, and the workspaces the kernels of a backward share.  A stage object has
// one such lane for the calls of its C ABI; bp_run_schedule gives every virtual device (up to
// kMaxLanes) a lane of its own, so that operations of different virtual devices, which are
// independent within a time slot (Section 3.3: at most one operation per device and slot), run side
// by side on the GPU.
constexpr int kMaxLanes = 4;
struct LaneState {
    hipStream_t stream = nullptr;
    // Weight-gradient GEMMs and the column reductions of the backward run on a second stream so
    // that their memory-bound tails overlap the next data-gradient kernels; events order the two.
    hipStream_t side = nullptr;
    hipEvent_t ev_ready[5] = {};         // main -> side: dz, du, dy, dqkv, da of the current layer
    hipEvent_t ev_layer_done[2] = {};    // side -> main: workspaces of layer parity p are free again
    bool layer_done_pending[2] = {false, false};
    hipEvent_t ev_misc = nullptr;        // side -> main: end of the previous backward call
    bool call_done_pending = false;
    // lean mode: forward scratch for a, m, g; per contraction segment the recomputed a, m, g and
    // throw-away LayerNorm statistics for the side stream's weight-gradient GEMMs
    void *fw_a = nullptr, *fw_m = nullptr, *fw_g = nullptr;
    void* re_x[3][kMaxGemmSegments] = {};    // [g | m | a][segment]
    float* re_stats = nullptr;
    std::vector<void*> pend_pool;                    // idle PendingMb buffers
    // backward workspaces; those the side stream reads exist once per layer parity, dx rotates
    // over three buffers (layer l writes l % 3, layer l-1 and its side work read it)
    void *ws_big1[2] = {}, *ws_big2[2] = {}, *ws_h1[2] = {}, *ws_h2[2] = {}, *ws_h5[2] = {};
    void *ws_h4 = nullptr, *ws_dx[3] = {};
    void* ws_gout = nullptr;             // private copy of a backward's grad_out (lanes only)
    float *ws_delta = nullptr, *ws_colsum[2] = {};
    float* ws_splitk = nullptr;          // split-K partials of main-stream GEMMs: 4 * T * H floats
    size_t ws_splitk_elems = 0;
    float* ws_splitk_side = nullptr;     // the same for the weight-gradient GEMMs of the side stream
    size_t ws_splitk_side_elems = 0;
    // bp_opts.forward_ahead: forwards run on a stream of their own, so that the forward of one
    // micro-batch overlaps the backward of another; it has its own split-K workspace
    hipStream_t fstream = nullptr;
    hipEvent_t ev_call = nullptr;        // main -> forward stream: everything enqueued before a forward call
    hipEvent_t ev_fwd_all = nullptr;     // forward stream -> main: every forward enqueued so far
    float* ws_splitk_fwd = nullptr;
};

struct Stage : LaneState {
    // shape
    int L = 0, H = 0, heads = 0, d = 0, S = 0, B = 0, T = 0, F = 0, n_chunks = 1;
    bool causal = true;
    int dtype = BP_BF16, max_inflight = 8;
    size_t esz = 2;
    float eps = 1e-5f;
    bool overlap = true;                 // false: everything on `stream` (also while timing kernels)
    bool forward_ahead = false;          // forwards on `fstream`

    // parameters (matrices in the storage dtype, vectors fp32) and fp32 gradients per direction
    void* params = nullptr;
    float* grads[2] = {nullptr, nullptr};
    // per (direction, chunk, layer): bit 0 set while the layer's weight-matrix gradients are
    // logically zero, bit 1 the same for its vector gradients (biases, LayerNorm).  The buffer
    // contents are then undefined and the next contribution overwrites them instead of adding,
    // which saves both the clearing pass and the first read of every read-modify-write.
    std::vector<uint8_t> grad_clean[2];
    // Grouped weight gradients: per (direction, chunk) the micro-batches waiting for their group.
    int wgrad_group = 1;
    bool lean = false;                   // stash without LN outputs and GELU output: recomputed for the weight gradients
    bool fuse_gelu = true;               // GELU forward/backward inside the GEMM epilogues when possible
    std::vector<PendGroup> pend[2];
    size_t q_dz = 0, q_du = 0, q_dy = 0, q_dqkv = 0, q_layer_bytes = 0;
    int slot_capacity = 8;                           // most live stashes (held ones come on top)
    // Each weight matrix is also kept transposed ([out,in]) so that the forward GEMMs read both
    // operands contraction-major like the data-gradient GEMMs do; slots BP_N_TENSORS.. hold them.
    size_t p_off[BP_N_TENSORS + 4], g_off[BP_N_TENSORS], p_layer_bytes = 0, g_layer_bytes = 0;

    // stash of one layer: byte offsets inside a slot
    size_t s_x, s_a, s_qkv, s_ctx, s_y, s_m, s_u, s_g, s_mean1, s_rstd1, s_mean2, s_rstd2, s_lse;
    size_t s_layer_bytes = 0;
    std::vector<StashSlot> slots;


    // key-padding lengths per micro-batch (device int32 [B])
    std::map<int, int32_t*> lens;

    // bp_run_schedule: one view of this object per lane.  A view shares the parameters and the
    // gradient buffers (it does not own them) and has its own lane, stash slots, weight-gradient
    // groups and clear flags: everything a (direction, stage) touches belongs to one virtual device,
    // hence to one lane, so the views never write the same memory or the same host state.
    bool is_view = false;
    int device = 0;                      // HIP device the object lives on
    std::vector<Stage*> views;
    bool copy_grad_out = false;          // backward copies grad_out first (its side stream must not read caller memory)
    int lane_alloc(LaneState& ln, bool with_stream);
    void lane_free(LaneState& ln, bool with_stream);
    int make_view(Stage** out);
    int run_lanes(const Layout& L, const bp_op* order, int n_ops, int D, int N, int lanes, const void* inputs,
                  const void* targets);
    std::vector<hipEvent_t> sched_ev;    // bp_run_schedule: completion event of every op of the order
    hipEvent_t ev_fork = nullptr;

    // buffers of bp_run_schedule, sized for sched_n micro-batches
    void *sched_act = nullptr, *sched_grad = nullptr;
    float* sched_loss = nullptr;
    int sched_n = 0;

    Prof prof;

    static int create(Stage** out, int layers, int hidden, int heads, int seq, int microbatch,
                      int causal, const bp_opts* opts);
    ~Stage();

    bool stream_valid() const { return true; }
    size_t tensor_elems(int id) const;
    static bool tensor_is_matrix(int id);
    void* param(int chunk, int layer, int id) const;
    void* param_t(int chunk, int layer, int id) const;   // transposed copy of a weight matrix
    static int transposed_slot(int id);
    float* grad(int dir, int chunk, int layer, int id) const;
    int check_tensor(int chunk, int layer, int id, size_t n) const;

    int set_param(int chunk, int layer, int id, const float* host, size_t n);
    int get_grad(int chunk, int layer, int id, float* host, size_t n);
    int zero_grad();
    int merge_directions();
    int set_seqlens(int mb, const int32_t* host);

    // activation memory in use: live stashes, stashes and output-gradient buffers kept by open
    // weight-gradient groups; peak of their sum since the last reset
    size_t peak_held_bytes = 0;
    void held_bytes(size_t out[3]) const;
    void note_held();
    int find_slot(int chunk, int mb) const;
    int acquire_slot(int chunk, int mb, int* out);
    int live_slots() const;

    int wgrad_one(int dir, int chunk, int l, int k, const void* cur_x, const void* cur_dy, int acc,
                  hipStream_t ss);
    int release_group(PendGroup& grp, hipStream_t ss);
    int flush_group(int dir, int chunk);
    int flush_all();
    int drop_pending();
    int gemm(const void* A, int lda, int a_t, const void* Bm, int ldb, int b_t, void* C, int ldc,
             int M, int N, int K, const float* bias, const void* residual, int accumulate,
             hipStream_t on = nullptr, bool use_on = false);
    hipStream_t side_stream() const { return (overlap && !prof.on && side) ? side : stream; }
    hipStream_t forward_stream() const { return (forward_ahead && !prof.on && fstream) ? fstream : stream; }
    int wait_forward();
    int sync_all();
    int forward(int chunk, int mb, const void* act_in, void* act_out);
    int backward(int chunk, int mb, const void* grad_out, void* grad_in, int dir);
    int run_schedule(const Layout& L, const bp_op* order, int n_ops, int D, const void* inputs,
                     const void* targets, float* loss_out);
};

// pure CPU schedule logic
int schedule_vmap(int dir, int stage, int D);
int schedule_vmap(const Layout& L, int dir, int stage, int D);
int schedule_validate(const Layout& L, const bp_op* order, int n_ops, int D, int N);

}  // namespace bp
