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

// Optional event timing of every launch, grouped by kernel class.
struct Prof {
    struct Pending { int kid; hipEvent_t start, stop; };
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
};

struct Stage {
    // shape
    int L = 0, H = 0, heads = 0, d = 0, S = 0, B = 0, T = 0, F = 0, n_chunks = 1;
    bool causal = true;
    int dtype = BP_BF16, max_inflight = 8;
    size_t esz = 2;
    float eps = 1e-5f;
    hipStream_t stream = nullptr;

    // parameters (matrices in the storage dtype, vectors fp32) and fp32 gradients per direction
    void* params = nullptr;
    float* grads[2] = {nullptr, nullptr};
    size_t p_off[BP_N_TENSORS], g_off[BP_N_TENSORS], p_layer_bytes = 0, g_layer_bytes = 0;

    // stash of one layer: byte offsets inside a slot
    size_t s_x, s_a, s_qkv, s_ctx, s_y, s_m, s_u, s_g, s_mean1, s_rstd1, s_mean2, s_rstd2, s_lse;
    size_t s_layer_bytes = 0;
    std::vector<StashSlot> slots;

    // backward workspaces
    void *ws_big1 = nullptr, *ws_big2 = nullptr, *ws_h1 = nullptr, *ws_h2 = nullptr, *ws_h3 = nullptr;
    float *ws_delta = nullptr, *ws_colsum = nullptr;

    // key-padding lengths per micro-batch (device int32 [B])
    std::map<int, int32_t*> lens;

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
    float* grad(int dir, int chunk, int layer, int id) const;
    int check_tensor(int chunk, int layer, int id, size_t n) const;

    int set_param(int chunk, int layer, int id, const float* host, size_t n);
    int get_grad(int chunk, int layer, int id, float* host, size_t n);
    int zero_grad();
    int merge_directions();
    int set_seqlens(int mb, const int32_t* host);

    int find_slot(int chunk, int mb) const;
    int acquire_slot(int chunk, int mb, int* out);
    int live_slots() const;

    int gemm(const void* A, int lda, int a_t, const void* Bm, int ldb, int b_t, void* C, int ldc,
             int M, int N, int K, const float* bias, const void* residual, int accumulate);
    int forward(int chunk, int mb, const void* act_in, void* act_out);
    int backward(int chunk, int mb, const void* grad_out, void* grad_in, int dir);
    int run_schedule(const bp_op* order, int n_ops, int D, const void* inputs, const void* targets,
                     float* loss_out);
};

// pure CPU schedule logic
int schedule_vmap(int dir, int stage, int D);
int schedule_validate(const bp_op* order, int n_ops, int D, int N);

}  // namespace bp
