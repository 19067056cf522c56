// Host side of the stage library: the stage object (weights, fp32 gradient accumulators per
// pipeline direction, activation stashes keyed by (chunk, micro-batch), backward workspaces),
// the forward / backward kernel sequences of a chunk, and the C ABI around them.
#include "bp_host.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>

namespace bp {

static thread_local std::string g_last_error;

int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return code;
}

const char* last_error() { return g_last_error.c_str(); }

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ------------------------------------------------------------------ shapes

size_t Stage::tensor_elems(int id) const {
    const size_t h = H, f = F;
    switch (id) {
        case BP_WQKV: return h * 3 * h;
        case BP_BQKV: return 3 * h;
        case BP_WO: return h * h;
        case BP_W1: return h * f;
        case BP_B1: return f;
        case BP_W2: return f * h;
        default: return h;   // LN vectors, bo, b2
    }
}

bool Stage::tensor_is_matrix(int id) { return id == BP_WQKV || id == BP_WO || id == BP_W1 || id == BP_W2; }

// ------------------------------------------------------------------ profiling

void Prof::begin(Stage* st, int kid, double flops, double bytes) {
    if (!on) return;
    hipEvent_t a, b;
    if (free_events.size() >= 2) {
        a = free_events.back(); free_events.pop_back();
        b = free_events.back(); free_events.pop_back();
    } else {
        hipEventCreate(&a);
        hipEventCreate(&b);
    }
    hipEventRecord(a, st->stream);
    pending.push_back({kid, a, b, kid == BP_K_GEMM ? next_shape : -1});
    next_shape = -1;
    flops_total[kid] += flops;
    bytes_total[kid] += bytes;
    launches[kid] += 1;
}

void Prof::end(Stage* st) {
    if (!on) return;
    hipEventRecord(pending.back().stop, st->stream);
}

void Prof::collect() {
    for (auto& p : pending) {
        float ms = 0.f;
        hipEventSynchronize(p.stop);
        hipEventElapsedTime(&ms, p.start, p.stop);
        ms_total[p.kid] += ms;
        if (p.shape >= 0) { shapes[p.shape].ms += ms; shapes[p.shape].launches += 1; }
        free_events.push_back(p.start);
        free_events.push_back(p.stop);
    }
    pending.clear();
}

void Prof::tag_gemm(int M, int N, int K, int a_t, int b_t, int nseg, int epi) {
    if (!on) return;
    const int d[7] = {M, N, K, a_t, b_t, nseg, epi};
    for (size_t i = 0; i < shapes.size(); ++i)
        if (!memcmp(shapes[i].dims, d, sizeof d)) { next_shape = (int)i; return; }
    ShapeStat ss{};
    memcpy(ss.dims, d, sizeof d);
    shapes.push_back(ss);
    next_shape = (int)shapes.size() - 1;
}

void Prof::reset() {
    collect();
    shapes.clear();
    for (int i = 0; i < BP_N_KERNEL_IDS; ++i) {
        ms_total[i] = 0; flops_total[i] = 0; bytes_total[i] = 0; launches[i] = 0;
    }
}

Prof::~Prof() {
    collect();
    for (auto e : free_events) hipEventDestroy(e);
}

struct Scoped {
    Stage* st;
    Scoped(Stage* s, int kid, double flops, double bytes) : st(s) { st->prof.begin(st, kid, flops, bytes); }
    ~Scoped() { st->prof.end(st); }
};

// ------------------------------------------------------------------ construction

static int dev_alloc(void** p, size_t bytes) {
    hipError_t e = hipMalloc(p, bytes ? bytes : 256);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(BP_ENOMEM, "hipMalloc(%zu bytes) failed: %s", bytes, hipGetErrorString(e));
    }
    return BP_OK;
}

int Stage::create(Stage** out, int layers, int hidden, int heads, int seq, int microbatch,
                  int causal, const bp_opts* o) {
    if (!out) return fail(BP_EINVAL, "out is null");
    if (layers <= 0 || hidden <= 0 || heads <= 0 || seq <= 0 || microbatch <= 0)
        return fail(BP_EINVAL, "layers, hidden, heads, seq, microbatch must be positive");
    if (hidden % heads) return fail(BP_ESHAPE, "hidden %d is not a multiple of heads %d", hidden, heads);
    const int d = hidden / heads;
    if (hidden % 8 || d % 8) return fail(BP_ESHAPE, "hidden and head dim must be multiples of 8");
    if (hidden > 8192) return fail(BP_ESHAPE, "hidden %d exceeds 8192", hidden);
    bp_opts opt;
    memset(&opt, 0, sizeof opt);
    opt.dtype = BP_BF16;
    if (o) opt = *o;
    if (opt.dtype != BP_F32 && opt.dtype != BP_BF16) return fail(BP_EINVAL, "unknown dtype %d", opt.dtype);
    if (opt.n_chunks < 0 || opt.mlp < 0 || opt.max_inflight < 0 || opt.ln_eps < 0)
        return fail(BP_EINVAL, "negative option");
    if (opt.stash_recompute != 0 && opt.stash_recompute != 1)
        return fail(BP_EINVAL, "stash_recompute %d is not 0 or 1", opt.stash_recompute);
    if (opt.wgrad_group < 0 || opt.wgrad_group > kMaxGemmSegments)
        return fail(BP_EINVAL, "wgrad_group %d outside 0..%d", opt.wgrad_group, kMaxGemmSegments);
    if (opt.forward_ahead != 0 && opt.forward_ahead != 1)
        return fail(BP_EINVAL, "forward_ahead %d is not 0 or 1", opt.forward_ahead);
    if (opt.mlp % 8) return fail(BP_ESHAPE, "mlp width must be a multiple of 8");
    if ((size_t)seq * sizeof(float) * 2 > 56000)
        return fail(BP_ESHAPE, "seq %d too long for the attention kernels", seq);

    Stage* st = new (std::nothrow) Stage();
    if (!st) return fail(BP_ENOMEM, "host allocation failed");
    st->L = layers; st->H = hidden; st->heads = heads; st->d = d; st->S = seq; st->B = microbatch;
    st->T = microbatch * seq;
    st->causal = causal != 0;
    st->n_chunks = opt.n_chunks ? opt.n_chunks : 1;
    st->F = opt.mlp ? opt.mlp : 4 * hidden;
    st->dtype = opt.dtype;
    st->max_inflight = opt.max_inflight ? opt.max_inflight : 8;
    st->eps = opt.ln_eps > 0 ? opt.ln_eps : 1e-5f;
    st->stream = (hipStream_t)opt.hip_stream;
    if (hipGetDevice(&st->device) != hipSuccess) { delete st; return fail(BP_EHIP, "hipGetDevice failed"); }
    st->esz = dtype_size(st->dtype);
    st->lean = opt.stash_recompute == 1;
    st->wgrad_group = opt.wgrad_group ? opt.wgrad_group : std::min(kMaxGemmSegments, std::max(1, 16384 / st->T));
    st->pend[0].resize(st->n_chunks);
    st->pend[1].resize(st->n_chunks);

    // parameter and gradient layout: one blob each, tensors 256-byte aligned
    size_t poff = 0, goff = 0;
    for (int t = 0; t < BP_N_TENSORS; ++t) {
        st->p_off[t] = poff;
        st->g_off[t] = goff;
        const size_t n = st->tensor_elems(t);
        poff += align_up(n * (tensor_is_matrix(t) ? st->esz : sizeof(float)), 256);
        goff += align_up(n * sizeof(float), 256);
    }
    for (int t = 0; t < BP_N_TENSORS; ++t) {
        if (!tensor_is_matrix(t)) continue;
        st->p_off[transposed_slot(t)] = poff;
        poff += align_up(st->tensor_elems(t) * st->esz, 256);
    }
    st->p_layer_bytes = poff;
    st->g_layer_bytes = goff;
    const size_t n_layers = (size_t)st->n_chunks * st->L;
    int rc;
    if ((rc = dev_alloc(&st->params, n_layers * poff))) { delete st; return rc; }
    for (int dir = 0; dir < 2; ++dir)
        if ((rc = dev_alloc((void**)&st->grads[dir], n_layers * goff))) { delete st; return rc; }

    // stash layout of one layer
    const size_t TH = (size_t)st->T * st->H * st->esz, TF = (size_t)st->T * st->F * st->esz;
    size_t so = 0;
    auto take = [&](size_t bytes) { size_t o = so; so += align_up(bytes, 256); return o; };
    // lean stash: a, m and g get no room (their offsets are never used then)
    st->s_x = take(TH); st->s_a = st->lean ? 0 : take(TH); st->s_qkv = take(3 * TH); st->s_ctx = take(TH);
    st->s_y = take(TH); st->s_m = st->lean ? 0 : take(TH); st->s_u = take(TF); st->s_g = st->lean ? 0 : take(TF);
    st->s_mean1 = take(st->T * sizeof(float)); st->s_rstd1 = take(st->T * sizeof(float));
    st->s_mean2 = take(st->T * sizeof(float)); st->s_rstd2 = take(st->T * sizeof(float));
    st->s_lse = take((size_t)st->B * st->heads * st->S * sizeof(float));
    st->s_layer_bytes = so;
    st->slots.resize(st->max_inflight);
    st->slot_capacity = st->max_inflight;
    so = 0;
    st->q_dz = take(TH); st->q_du = take(TF); st->q_dy = take(TH); st->q_dqkv = take(3 * TH);
    st->q_layer_bytes = so;

    // lane 0: workspaces, the second stream (default priority, not synchronising with the null
    // stream) and the events that order the two
    if ((rc = st->lane_alloc(*st, false))) { delete st; return rc; }
    if (opt.forward_ahead) {    // the forward stream, its two events and its split-K workspace
        hipError_t fe = hipStreamCreateWithFlags(&st->fstream, hipStreamNonBlocking);
        if (fe == hipSuccess) fe = hipEventCreateWithFlags(&st->ev_call, hipEventDisableTiming);
        if (fe == hipSuccess) fe = hipEventCreateWithFlags(&st->ev_fwd_all, hipEventDisableTiming);
        if (fe != hipSuccess) {
            delete st;
            return fail(BP_EHIP, "creating the forward stream failed: %s", hipGetErrorString(fe));
        }
        if (st->ws_splitk_elems &&
            (rc = dev_alloc((void**)&st->ws_splitk_fwd, st->ws_splitk_elems * sizeof(float)))) { delete st; return rc; }
        st->forward_ahead = true;
    }

    // initial values: zeros, LN gamma = 1
    hipError_t e = hipMemsetAsync(st->params, 0, n_layers * poff, st->stream);
    if (e == hipSuccess) e = launch_fill_f32(st->grads[0], n_layers * goff / 4, 0.f, st->stream);
    if (e == hipSuccess) e = launch_fill_f32(st->grads[1], n_layers * goff / 4, 0.f, st->stream);
    st->grad_clean[0].assign(n_layers, 3);
    st->grad_clean[1].assign(n_layers, 3);
    for (int c = 0; c < st->n_chunks && e == hipSuccess; ++c)
        for (int l = 0; l < st->L && e == hipSuccess; ++l) {
            e = launch_fill_f32((float*)st->param(c, l, BP_LN1_G), st->H, 1.f, st->stream);
            if (e == hipSuccess) e = launch_fill_f32((float*)st->param(c, l, BP_LN2_G), st->H, 1.f, st->stream);
        }
    if (e == hipSuccess) e = hipStreamSynchronize(st->stream);
    if (e != hipSuccess) {
        delete st;
        return fail(BP_EHIP, "initialisation failed: %s", hipGetErrorString(e));
    }
    *out = st;
    return BP_OK;
}

int Stage::lane_alloc(LaneState& ln, bool with_stream) {
    const size_t TH = (size_t)T * H * esz, TF = (size_t)T * F * esz;
    const size_t big = std::max((size_t)F, (size_t)3 * H);
    int rc = BP_OK;
    for (int p = 0; p < 2 && !rc; ++p) {
        (rc = dev_alloc(&ln.ws_big1[p], (size_t)T * big * esz)) ||
            (rc = dev_alloc(&ln.ws_big2[p], (size_t)T * 3 * H * esz)) ||
            (rc = dev_alloc(&ln.ws_h1[p], TH)) || (rc = dev_alloc(&ln.ws_h2[p], TH)) ||
            (rc = dev_alloc(&ln.ws_h5[p], TH)) ||
            (rc = dev_alloc((void**)&ln.ws_colsum[p],
                            std::max<size_t>(colsum_chunks(T) * ((size_t)9 * H + F), 1024) * sizeof(float)));
    }
    for (int i = 0; i < 3 && !rc; ++i) rc = dev_alloc(&ln.ws_dx[i], TH);
    if (!rc) rc = dev_alloc(&ln.ws_h4, TH);
    if (!rc) rc = dev_alloc(&ln.ws_gout, TH);
    if (!rc && dtype == BP_BF16) {
        ln.ws_splitk_elems = (size_t)4 * T * H;
        rc = dev_alloc((void**)&ln.ws_splitk, ln.ws_splitk_elems * sizeof(float));
        // weight gradients with few output tiles (H x H, or a narrow MLP) and a long token axis
        ln.ws_splitk_side_elems = std::min((size_t)4 * H * std::max(H, F), (size_t)64 << 20);
        if (!rc) rc = dev_alloc((void**)&ln.ws_splitk_side, ln.ws_splitk_side_elems * sizeof(float));
    }
    if (!rc && lean) {
        (rc = dev_alloc(&ln.fw_a, TH)) || (rc = dev_alloc(&ln.fw_m, TH)) || (rc = dev_alloc(&ln.fw_g, TF)) ||
            (rc = dev_alloc((void**)&ln.re_stats, (size_t)2 * T * sizeof(float)));
        for (int i = 0; i < kMaxGemmSegments && !rc; ++i)
            (rc = dev_alloc(&ln.re_x[0][i], TF)) || (rc = dev_alloc(&ln.re_x[1][i], TH)) ||
                (rc = dev_alloc(&ln.re_x[2][i], TH));
    }
    if (!rc) rc = dev_alloc((void**)&ln.ws_delta, (size_t)B * heads * S * sizeof(float));
    if (rc) return rc;
    hipError_t e = hipSuccess;
    if (with_stream) e = hipStreamCreateWithFlags(&ln.stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&ln.side, hipStreamNonBlocking);
    for (int i = 0; i < 5 && e == hipSuccess; ++i) e = hipEventCreateWithFlags(&ln.ev_ready[i], hipEventDisableTiming);
    for (int i = 0; i < 2 && e == hipSuccess; ++i) e = hipEventCreateWithFlags(&ln.ev_layer_done[i], hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ln.ev_misc, hipEventDisableTiming);
    if (e != hipSuccess) return fail(BP_EHIP, "creating a lane's streams and events failed: %s", hipGetErrorString(e));
    return BP_OK;
}

void Stage::lane_free(LaneState& ln, bool with_stream) {
    if (ln.side) { hipStreamSynchronize(ln.side); hipStreamDestroy(ln.side); }
    if (with_stream && ln.stream) { hipStreamSynchronize(ln.stream); hipStreamDestroy(ln.stream); }
    if (ln.fstream) { hipStreamSynchronize(ln.fstream); hipStreamDestroy(ln.fstream); }
    if (ln.ev_call) hipEventDestroy(ln.ev_call);
    if (ln.ev_fwd_all) hipEventDestroy(ln.ev_fwd_all);
    hipFree(ln.ws_splitk_fwd);
    for (auto e : ln.ev_ready) if (e) hipEventDestroy(e);
    for (auto e : ln.ev_layer_done) if (e) hipEventDestroy(e);
    if (ln.ev_misc) hipEventDestroy(ln.ev_misc);
    for (auto b : ln.pend_pool) hipFree(b);
    for (int p = 0; p < 2; ++p) {
        hipFree(ln.ws_big1[p]); hipFree(ln.ws_big2[p]); hipFree(ln.ws_h1[p]); hipFree(ln.ws_h2[p]); hipFree(ln.ws_h5[p]);
        hipFree(ln.ws_colsum[p]);
    }
    for (auto b : ln.ws_dx) hipFree(b);
    hipFree(ln.ws_h4); hipFree(ln.ws_gout);
    hipFree(ln.ws_splitk); hipFree(ln.ws_splitk_side);
    hipFree(ln.fw_a); hipFree(ln.fw_m); hipFree(ln.fw_g); hipFree(ln.re_stats);
    for (auto& row : ln.re_x) for (auto b : row) hipFree(b);
    hipFree(ln.ws_delta);
}

// A view for one lane of bp_run_schedule: same shape, shared parameters and gradient buffers, own
// lane (with a stream of its own), stash slots, groups and clear flags.
int Stage::make_view(Stage** out) {
    Stage* v = new (std::nothrow) Stage();
    if (!v) return fail(BP_ENOMEM, "host allocation failed");
    v->is_view = true;
    v->device = device;
    v->L = L; v->H = H; v->heads = heads; v->d = d; v->S = S; v->B = B; v->T = T; v->F = F; v->n_chunks = n_chunks;
    v->causal = causal; v->dtype = dtype; v->max_inflight = max_inflight; v->esz = esz; v->eps = eps;
    v->overlap = overlap; v->params = params; v->grads[0] = grads[0]; v->grads[1] = grads[1];
    v->wgrad_group = wgrad_group; v->lean = lean; v->fuse_gelu = fuse_gelu;
    v->q_dz = q_dz; v->q_du = q_du; v->q_dy = q_dy; v->q_dqkv = q_dqkv; v->q_layer_bytes = q_layer_bytes;
    memcpy(v->p_off, p_off, sizeof p_off); memcpy(v->g_off, g_off, sizeof g_off);
    v->p_layer_bytes = p_layer_bytes; v->g_layer_bytes = g_layer_bytes;
    v->s_x = s_x; v->s_a = s_a; v->s_qkv = s_qkv; v->s_ctx = s_ctx; v->s_y = s_y; v->s_m = s_m; v->s_u = s_u; v->s_g = s_g;
    v->s_mean1 = s_mean1; v->s_rstd1 = s_rstd1; v->s_mean2 = s_mean2; v->s_rstd2 = s_rstd2; v->s_lse = s_lse;
    v->s_layer_bytes = s_layer_bytes;
    v->slots.resize(max_inflight);
    v->slot_capacity = slot_capacity;
    v->pend[0].resize(n_chunks);
    v->pend[1].resize(n_chunks);
    v->grad_clean[0].assign(grad_clean[0].size(), 3);
    v->grad_clean[1].assign(grad_clean[1].size(), 3);
    int rc = v->lane_alloc(*v, true);
    if (rc) { delete v; return rc; }
    *out = v;
    return BP_OK;
}

int Stage::sync_all() {
    hipError_t e = hipStreamSynchronize(stream);
    if (e == hipSuccess && side) e = hipStreamSynchronize(side);
    if (e == hipSuccess && fstream) e = hipStreamSynchronize(fstream);
    if (e != hipSuccess) return fail(BP_EHIP, "synchronise: %s", hipGetErrorString(e));
    for (Stage* v : views) {
        int rc = v->sync_all();
        if (rc) return rc;
    }
    return BP_OK;
}

Stage::~Stage() {
    sync_all();
    for (Stage* v : views) delete v;
    lane_free(*this, is_view);
    if (!is_view) {
        hipFree(params);
        hipFree(grads[0]);
        hipFree(grads[1]);
        for (auto& kv : lens) hipFree(kv.second);
    }
    for (auto& s : slots) {
        hipFree(s.buf);
        if (s.side_done) hipEventDestroy(s.side_done);
        if (s.fwd_done) hipEventDestroy(s.fwd_done);
    }
    for (int dir = 0; dir < 2; ++dir)
        for (auto& grp : pend[dir])
            for (auto& it : grp.items) hipFree(it.buf);
    for (auto e : sched_ev) if (e) hipEventDestroy(e);
    if (ev_fork) hipEventDestroy(ev_fork);
    hipFree(sched_act); hipFree(sched_grad); hipFree(sched_loss);
}

int Stage::transposed_slot(int id) {
    return BP_N_TENSORS + (id == BP_WQKV ? 0 : id == BP_WO ? 1 : id == BP_W1 ? 2 : 3);
}
void* Stage::param_t(int chunk, int layer, int id) const {
    return (char*)params + ((size_t)chunk * L + layer) * p_layer_bytes + p_off[transposed_slot(id)];
}
void* Stage::param(int chunk, int layer, int id) const {
    return (char*)params + ((size_t)chunk * L + layer) * p_layer_bytes + p_off[id];
}
float* Stage::grad(int dir, int chunk, int layer, int id) const {
    return (float*)((char*)grads[dir] + ((size_t)chunk * L + layer) * g_layer_bytes + g_off[id]);
}

// ------------------------------------------------------------------ parameters and gradients

int Stage::check_tensor(int chunk, int layer, int id, size_t n) const {
    if (chunk < 0 || chunk >= n_chunks) return fail(BP_EINVAL, "chunk %d out of range [0,%d)", chunk, n_chunks);
    if (layer < 0 || layer >= L) return fail(BP_EINVAL, "layer %d out of range [0,%d)", layer, L);
    if (id < 0 || id >= BP_N_TENSORS) return fail(BP_EINVAL, "tensor id %d out of range", id);
    if (n != tensor_elems(id))
        return fail(BP_ESHAPE, "tensor %d has %zu elements, got %zu", id, tensor_elems(id), n);
    return BP_OK;
}

int Stage::set_param(int chunk, int layer, int id, const float* host, size_t n) {
    int rc = check_tensor(chunk, layer, id, n);
    if (rc) return rc;
    if (!host) return fail(BP_EINVAL, "host pointer is null");
    if ((rc = wait_forward())) return rc;    // a forward still in flight reads the old values
    void* dst = param(chunk, layer, id);
    hipError_t e;
    // rows x cols of the [in, out] matrix
    const int rows = id == BP_W2 ? F : H;
    const int cols = id == BP_WQKV ? 3 * H : id == BP_W1 ? F : H;
    if (!tensor_is_matrix(id) || dtype == BP_F32) {
        e = hipMemcpyAsync(dst, host, n * sizeof(float), hipMemcpyHostToDevice, stream);
        if (e == hipSuccess && tensor_is_matrix(id))
            e = launch_transpose(dtype, rows, cols, dst, param_t(chunk, layer, id), stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
    } else {
        float* tmp = nullptr;
        if ((rc = dev_alloc((void**)&tmp, n * sizeof(float)))) return rc;
        e = hipMemcpyAsync(tmp, host, n * sizeof(float), hipMemcpyHostToDevice, stream);
        if (e == hipSuccess) e = launch_cast_from_f32(dtype, tmp, dst, n, stream);
        if (e == hipSuccess) e = launch_transpose(dtype, rows, cols, dst, param_t(chunk, layer, id), stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        hipFree(tmp);
    }
    if (e != hipSuccess) return fail(BP_EHIP, "set_param: %s", hipGetErrorString(e));
    return BP_OK;
}

int Stage::get_grad(int chunk, int layer, int id, float* host, size_t n) {
    int rc = check_tensor(chunk, layer, id, n);
    if (rc) return rc;
    if (!host) return fail(BP_EINVAL, "host pointer is null");
    if ((rc = flush_all())) return rc;
    if ((rc = sync_all())) return rc;
    if (grad_clean[0][(size_t)chunk * L + layer] & (tensor_is_matrix(id) ? 1 : 2)) {   // nothing since the last clear
        memset(host, 0, n * sizeof(float));
        return BP_OK;
    }
    hipError_t e = hipMemcpyAsync(host, grad(0, chunk, layer, id), n * sizeof(float),
                                  hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail(BP_EHIP, "get_grad: %s", hipGetErrorString(e));
    return BP_OK;
}

int Stage::zero_grad() {
    // host bookkeeping only: kernels enqueued before this call still add into the old contents,
    // kernels enqueued after it see the layer as clear and overwrite.  Weight gradients still
    // waiting for their group belong to what is being cleared and are dropped.
    int rc = drop_pending();
    if (rc) return rc;
    grad_clean[0].assign(grad_clean[0].size(), 3);
    grad_clean[1].assign(grad_clean[1].size(), 3);
    return BP_OK;
}

int Stage::merge_directions() {
    int rc = flush_all();
    if (rc) return rc;
    const size_t n = g_layer_bytes / sizeof(float);
    Scoped sc(this, BP_K_OTHER, 0, 0);
    // every writer of the gradient buffers runs on the side stream, so the merge goes there too
    hipStream_t gs = side_stream();
    for (size_t i = 0; i < grad_clean[0].size(); ++i) {
        const int c0 = grad_clean[0][i], c1 = grad_clean[1][i];
        if (c1 == 3) continue;
        if (c1 != 0 || (c0 != 0 && c0 != 3))
            return fail(BP_ESTATE, "merge_directions: layer %zu is partly written", i);
        float* g0 = (float*)((char*)grads[0] + i * g_layer_bytes);
        float* g1 = (float*)((char*)grads[1] + i * g_layer_bytes);
        hipError_t e = c0 == 3 ? hipMemcpyAsync(g0, g1, g_layer_bytes, hipMemcpyDeviceToDevice, gs)
                               : launch_add_f32(g0, g1, n, gs);
        if (e != hipSuccess) return fail(BP_EHIP, "merge_directions: %s", hipGetErrorString(e));
        grad_clean[0][i] = 0;
        grad_clean[1][i] = 3;
    }
    return BP_OK;
}

// ------------------------------------------------------------------ grouped weight gradients

// Gradient of weight matrix k (0: W2, 1: W1, 2: Wo, 3: Wqkv) of one layer over the group's waiting
// micro-batches plus, when cur_x (the current micro-batch's stash of this layer) is given, the
// current one: a single GEMM whose contraction runs over all their tokens.
int Stage::wgrad_one(int dir, int chunk, int l, int k, const void* cur_x, const void* cur_dy, int acc,
                     hipStream_t ss) {
    static const int ids[4] = {BP_W2, BP_W1, BP_WO, BP_WQKV};
    const size_t sx[4] = {s_g, s_m, s_ctx, s_a}, qy[4] = {q_dz, q_du, q_dy, q_dqkv};
    const int Mk[4] = {F, H, H, H}, Nk[4] = {H, F, H, 3 * H};
    const PendGroup& grp = pend[dir][chunk];
    const void* xs[kMaxGemmSegments];
    const void* ys[kMaxGemmSegments];
    int n = 0;
    // Lean stash: the operand of W2, W1 and Wqkv (GELU output, LN2 output, LN1 output) was not
    // kept; it is rebuilt from the stashed u, y, x on this stream right before the GEMM.
    auto operand = [&](const char* stash_layer, int seg, const void** out) -> int {
        if (!lean || k == 2) { *out = stash_layer + sx[k]; return BP_OK; }
        const int which = k == 0 ? 0 : k == 1 ? 1 : 2;
        void* dst = re_x[which][seg];
        hipError_t e;
        if (k == 0) {
            Scoped sc(this, BP_K_GELU_FWD, 0, 2.0 * T * F * esz);
            e = launch_gelu_fwd(dtype, T, F, stash_layer + s_u, (const float*)param(chunk, l, BP_B1), dst, ss);
        } else {
            Scoped sc(this, BP_K_LN_FWD, 0, 2.0 * T * H * esz);
            const bool second = k == 1;
            e = launch_ln_fwd(dtype, T, H, stash_layer + (second ? s_y : s_x),
                              (const float*)param(chunk, l, second ? BP_LN2_G : BP_LN1_G),
                              (const float*)param(chunk, l, second ? BP_LN2_B : BP_LN1_B), eps, dst,
                              re_stats, re_stats + T, nullptr, ss);
        }
        if (e != hipSuccess) return fail(BP_EHIP, "recomputing a stash tensor: %s", hipGetErrorString(e));
        *out = dst;
        return BP_OK;
    };
    int rc;
    for (const PendingMb& it : grp.items) {
        if (n >= kMaxGemmSegments) return fail(BP_ESTATE, "weight-gradient group overflow");
        if ((rc = operand((const char*)slots[it.slot].buf + (size_t)l * s_layer_bytes, n, &xs[n]))) return rc;
        ys[n] = (const char*)it.buf + (size_t)l * q_layer_bytes + qy[k];
        ++n;
    }
    if (cur_x) {
        if (n >= kMaxGemmSegments) return fail(BP_ESTATE, "weight-gradient group overflow");
        if ((rc = operand((const char*)cur_x, n, &xs[n]))) return rc;
        ys[n] = cur_dy; ++n;
    }
    if (n == 0) return BP_OK;
    GemmArgs g;
    g.A = xs[0]; g.B = ys[0]; g.C = grad(dir, chunk, l, ids[k]); g.bias = nullptr; g.residual = nullptr;
    g.M = Mk[k]; g.N = Nk[k]; g.K = T; g.lda = Mk[k]; g.ldb = Nk[k]; g.ldc = Nk[k];
    g.a_t = 1; g.b_t = 0; g.accumulate = acc;
    g.nseg = n;
    for (int i = 1; i < n; ++i) { g.A_more[i - 1] = xs[i]; g.B_more[i - 1] = ys[i]; }
    // all weight-gradient GEMMs run on one stream (the side stream, or the main one when the two
    // are merged), one after the other, so they can share one split-K workspace
    g.split_ws = ws_splitk_side;
    g.split_ws_elems = ws_splitk_side_elems;
    prof.tag_gemm(Mk[k], Nk[k], T, 1, 0, n, 0);
    Scoped sc(this, BP_K_GEMM, 2.0 * Mk[k] * Nk[k] * (double)T * n, 0);
    hipError_t e = launch_gemm(dtype, g, ss);
    if (e != hipSuccess) return fail(BP_EHIP, "weight-gradient GEMM: %s", hipGetErrorString(e));
    return BP_OK;
}

// The group's stashes and buffers become reusable once the side stream has passed this point.
int Stage::release_group(PendGroup& grp, hipStream_t ss) {
    for (PendingMb& it : grp.items) {
        StashSlot& sl = slots[it.slot];
        if (ss != stream) {
            hipError_t e = hipSuccess;
            if (!sl.side_done) e = hipEventCreateWithFlags(&sl.side_done, hipEventDisableTiming);
            if (e == hipSuccess) e = hipEventRecord(sl.side_done, ss);
            if (e != hipSuccess) return fail(BP_EHIP, "release_group: %s", hipGetErrorString(e));
            sl.side_pending = true;
        }
        sl.held = false;
        pend_pool.push_back(it.buf);
    }
    grp.items.clear();
    return BP_OK;
}

int Stage::flush_group(int dir, int chunk) {
    PendGroup& grp = pend[dir][chunk];
    if (grp.items.empty()) return BP_OK;
    hipStream_t ss = side_stream();
    if (ss != stream) {     // the waiting gradients were written on the main stream
        hipError_t e = hipEventRecord(ev_ready[0], stream);
        if (e == hipSuccess) e = hipStreamWaitEvent(ss, ev_ready[0], 0);
        if (e != hipSuccess) return fail(BP_EHIP, "flush_group: %s", hipGetErrorString(e));
    }
    int rc;
    for (int l = L - 1; l >= 0; --l) {
        uint8_t& clean = grad_clean[dir][(size_t)chunk * L + l];
        for (int k = 0; k < 4; ++k)
            if ((rc = wgrad_one(dir, chunk, l, k, nullptr, nullptr, (clean & 1) ? 2 : 1, ss))) return rc;
        clean &= ~1;
    }
    if ((rc = release_group(grp, ss))) return rc;
    if (ss != stream) {     // the next backward must not overwrite buffers these GEMMs still read
        hipError_t e = hipEventRecord(ev_misc, ss);
        if (e != hipSuccess) return fail(BP_EHIP, "flush_group: %s", hipGetErrorString(e));
        call_done_pending = true;
    }
    return BP_OK;
}

int Stage::flush_all() {
    for (int dir = 0; dir < 2; ++dir)
        for (int c = 0; c < n_chunks; ++c) {
            int rc = flush_group(dir, c);
            if (rc) return rc;
        }
    return BP_OK;
}

int Stage::drop_pending() {
    hipStream_t ss = side_stream();
    for (int dir = 0; dir < 2; ++dir)
        for (auto& grp : pend[dir]) {
            int rc = release_group(grp, ss);      // column sums of those calls may still be running
            if (rc) return rc;
        }
    return BP_OK;
}

int Stage::set_seqlens(int mb, const int32_t* host) {
    if (mb < 0) return fail(BP_EINVAL, "mb %d is negative", mb);
    if (causal) return fail(BP_ESTATE, "key padding lengths on a causal stage");
    for (auto& s : slots)
        if (s.live && s.mb == mb) return fail(BP_ESTATE, "micro-batch %d has a live stash", mb);
    auto it = lens.find(mb);
    if (!host) {
        if (it != lens.end()) {
            hipStreamSynchronize(stream);
            hipFree(it->second);
            lens.erase(it);
        }
        return BP_OK;
    }
    for (int b = 0; b < B; ++b)
        if (host[b] < 1 || host[b] > S) return fail(BP_EINVAL, "length %d outside 1..%d", host[b], S);
    int32_t* dev = nullptr;
    if (it != lens.end()) dev = it->second;
    else {
        int rc = dev_alloc((void**)&dev, B * sizeof(int32_t));
        if (rc) return rc;
        lens[mb] = dev;
    }
    if (int rc = wait_forward()) return rc;  // a forward still in flight reads the old lengths
    hipError_t e = hipMemcpyAsync(dev, host, B * sizeof(int32_t), hipMemcpyHostToDevice, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail(BP_EHIP, "set_seqlens: %s", hipGetErrorString(e));
    return BP_OK;
}

// ------------------------------------------------------------------ stash slots

void Stage::held_bytes(size_t out[3]) const {
    out[0] = out[1] = out[2] = 0;
    for (const auto& sl : slots) {
        if (sl.live) out[0] += (size_t)L * s_layer_bytes;
        else if (sl.held) out[1] += (size_t)L * s_layer_bytes;
    }
    for (int dir = 0; dir < 2; ++dir)
        for (const auto& grp : pend[dir]) out[2] += grp.items.size() * (size_t)L * q_layer_bytes;
}

void Stage::note_held() {
    size_t h[3];
    held_bytes(h);
    peak_held_bytes = std::max(peak_held_bytes, h[0] + h[1] + h[2]);
}

int Stage::find_slot(int chunk, int mb) const {
    for (size_t i = 0; i < slots.size(); ++i)
        if (slots[i].live && slots[i].chunk == chunk && slots[i].mb == mb) return (int)i;
    return -1;
}

int Stage::acquire_slot(int chunk, int mb, int* out) {
    if (find_slot(chunk, mb) >= 0)
        return fail(BP_ESTATE, "forward(chunk %d, mb %d) while its stash is still live", chunk, mb);
    int live = 0, pick = -1;
    for (size_t i = 0; i < slots.size(); ++i) {
        live += slots[i].live;
        if (pick < 0 && !slots[i].live && !slots[i].held) pick = (int)i;
    }
    if (live >= slot_capacity)
        return fail(BP_ESTATE, "all %d stash slots are live (max_inflight)", slot_capacity);
    if (pick < 0) {         // every idle slot is held by a weight-gradient group: add one
        slots.emplace_back();
        pick = (int)slots.size() - 1;
    }
    StashSlot& sl = slots[pick];
    if (!sl.buf) {
        int rc = dev_alloc(&sl.buf, (size_t)L * s_layer_bytes);
        if (rc) return rc;
    }
    if (sl.side_pending) {
        // the previous owner's weight-gradient kernels may still be reading this stash
        hipError_t e = hipStreamWaitEvent(forward_stream(), sl.side_done, 0);
        if (e != hipSuccess) return fail(BP_EHIP, "stash reuse wait: %s", hipGetErrorString(e));
        sl.side_pending = false;
    }

    sl.live = true; sl.chunk = chunk; sl.mb = mb;
    *out = pick;
    return BP_OK;
}

// ------------------------------------------------------------------ forward of one chunk

#define BP_LAUNCH(expr)                                                                 \
    do {                                                                                \
        hipError_t e_ = (expr);                                                         \
        if (e_ != hipSuccess) return fail(BP_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

int Stage::gemm(const void* A, int lda, int a_t, const void* Bm, int ldb, int b_t, void* C, int ldc,
                int M, int N, int K, const float* bias, const void* residual, int accumulate,
                hipStream_t on, bool use_on) {
    GemmArgs g;
    g.A = A; g.B = Bm; g.C = C; g.bias = bias; g.residual = residual;
    g.M = M; g.N = N; g.K = K; g.lda = lda; g.ldb = ldb; g.ldc = ldc;
    g.a_t = a_t; g.b_t = b_t; g.accumulate = accumulate;
    if (!use_on || on == stream) {      // one split-K workspace per stream: the main stream's ...
        g.split_ws = ws_splitk;
        g.split_ws_elems = ws_splitk_elems;
    } else if (on == fstream && ws_splitk_fwd) {    // ... and the forward stream's
        g.split_ws = ws_splitk_fwd;
        g.split_ws_elems = ws_splitk_elems;
    }
    prof.tag_gemm(M, N, K, a_t, b_t, 1, 0);
    Scoped sc(this, BP_K_GEMM, 2.0 * M * N * K, 0);
    BP_LAUNCH(launch_gemm(dtype, g, use_on ? on : stream));
    return BP_OK;
}

int Stage::forward(int chunk, int mb, const void* act_in, void* act_out) {
    if (chunk < 0 || chunk >= n_chunks) return fail(BP_EINVAL, "chunk %d out of range [0,%d)", chunk, n_chunks);
    if (mb < 0) return fail(BP_EINVAL, "mb %d is negative", mb);
    if (!act_in || !act_out) return fail(BP_EINVAL, "activation pointer is null");
    if (act_in == act_out) return fail(BP_EINVAL, "act_in and act_out must not overlap");
    int slot, rc;
    // With forward_ahead the call runs on the forward stream, behind everything the stage's stream
    // holds at this moment (the caller's producer of act_in, parameter updates, earlier calls);
    // backwards enqueued later run beside it.
    const hipStream_t fs = forward_stream();
    if (fs != stream) {
        BP_LAUNCH(hipEventRecord(ev_call, stream));
        BP_LAUNCH(hipStreamWaitEvent(fs, ev_call, 0));
    }
    if ((rc = acquire_slot(chunk, mb, &slot))) return rc;
    note_held();
    auto it = lens.find(mb);
    const int32_t* ln = it == lens.end() ? nullptr : it->second;
    const double unit = (double)T * H * esz;   // bytes of one [T,H] tensor
    const double attn_c = causal ? 0.5 : 1.0;

    for (int l = 0; l < L; ++l) {
        char* sb = (char*)slots[slot].buf + (size_t)l * s_layer_bytes;
        const void* x = l == 0 ? act_in : (const void*)(sb + s_x);
        void* z = l == L - 1 ? act_out : (void*)(sb + s_layer_bytes + s_x);
        // LN outputs and GELU output: kept in the stash, or scratch when they are recomputed later
        void* a_out = lean ? fw_a : (void*)(sb + s_a);
        void* m_out = lean ? fw_m : (void*)(sb + s_m);
        void* g_out = lean ? fw_g : (void*)(sb + s_g);
        {   // a = LN1(x); layer 0 also keeps a copy of the caller's input for the backward
            Scoped sc(this, BP_K_LN_FWD, 0, 2 * unit);
            BP_LAUNCH(launch_ln_fwd(dtype, T, H, x, (const float*)param(chunk, l, BP_LN1_G),
                                    (const float*)param(chunk, l, BP_LN1_B), eps, a_out,
                                    (float*)(sb + s_mean1), (float*)(sb + s_rstd1),
                                    l == 0 ? sb + s_x : nullptr, fs));
        }
        if ((rc = gemm(a_out, H, 0, param_t(chunk, l, BP_WQKV), H, 1, sb + s_qkv, 3 * H, T, 3 * H, H,
                       (const float*)param(chunk, l, BP_BQKV), nullptr, 0, fs, true))) return rc;
        {
            AttnArgs a{B, S, heads, d, causal ? 1 : 0, ln, sb + s_qkv, sb + s_ctx, (float*)(sb + s_lse),
                       nullptr, nullptr, nullptr};
            Scoped sc(this, BP_K_ATTN_FWD, 4.0 * T * S * H * attn_c, 0);
            BP_LAUNCH(launch_attn_fwd(dtype, a, fs));
        }
        if ((rc = gemm(sb + s_ctx, H, 0, param_t(chunk, l, BP_WO), H, 1, sb + s_y, H, T, H, H,
                       (const float*)param(chunk, l, BP_BO), x, 0, fs, true))) return rc;
        {
            Scoped sc(this, BP_K_LN_FWD, 0, 2 * unit);
            BP_LAUNCH(launch_ln_fwd(dtype, T, H, sb + s_y, (const float*)param(chunk, l, BP_LN2_G),
                                    (const float*)param(chunk, l, BP_LN2_B), eps, m_out,
                                    (float*)(sb + s_mean2), (float*)(sb + s_rstd2), nullptr, fs));
        }
        {   // u = m W1 and g = gelu(u + b1): one kernel when the GEMM can carry the activation
            GemmArgs fg;
            fg.A = m_out; fg.B = param_t(chunk, l, BP_W1); fg.C = sb + s_u;
            fg.bias = (const float*)param(chunk, l, BP_B1); fg.residual = nullptr;
            fg.M = T; fg.N = F; fg.K = H; fg.lda = H; fg.ldb = H; fg.ldc = F;
            fg.a_t = 0; fg.b_t = 1; fg.accumulate = 0;
            fg.epi = EPI_GELU_FWD; fg.C2 = g_out;
            if (fuse_gelu && gemm_can_fuse_epilogue(dtype, fg)) {
                prof.tag_gemm(T, F, H, 0, 1, 1, EPI_GELU_FWD);
                Scoped sc(this, BP_K_GEMM, 2.0 * T * (double)F * H, 0);
                BP_LAUNCH(launch_gemm(dtype, fg, fs));
            } else {
                if ((rc = gemm(m_out, H, 0, param_t(chunk, l, BP_W1), H, 1, sb + s_u, F, T, F, H, nullptr,
                               nullptr, 0, fs, true))) return rc;
                Scoped sc(this, BP_K_GELU_FWD, 0, 2.0 * T * F * esz);
                BP_LAUNCH(launch_gelu_fwd(dtype, T, F, sb + s_u, (const float*)param(chunk, l, BP_B1),
                                          g_out, fs));
            }
        }
        if ((rc = gemm(g_out, F, 0, param_t(chunk, l, BP_W2), F, 1, z, H, T, H, F,
                       (const float*)param(chunk, l, BP_B2), sb + s_y, 0, fs, true))) return rc;
    }
    if (fs != stream) {     // the backward of this micro-batch (on the stage's stream) waits for this
        StashSlot& sl = slots[slot];
        if (!sl.fwd_done) BP_LAUNCH(hipEventCreateWithFlags(&sl.fwd_done, hipEventDisableTiming));
        BP_LAUNCH(hipEventRecord(sl.fwd_done, fs));
        sl.fwd_pending = true;
    }
    return BP_OK;
}

// The stage's stream waits for every forward enqueued so far (forward_ahead; a no-op otherwise).
int Stage::wait_forward() {
    if (!fstream) return BP_OK;
    hipError_t e = hipEventRecord(ev_fwd_all, fstream);
    if (e == hipSuccess) e = hipStreamWaitEvent(stream, ev_fwd_all, 0);
    if (e != hipSuccess) return fail(BP_EHIP, "wait for the forward stream: %s", hipGetErrorString(e));
    for (auto& sl : slots) sl.fwd_pending = false;
    return BP_OK;
}

// ------------------------------------------------------------------ backward of one chunk

int Stage::backward(int chunk, int mb, const void* grad_out, void* grad_in, int dir) {
    if (chunk < 0 || chunk >= n_chunks) return fail(BP_EINVAL, "chunk %d out of range [0,%d)", chunk, n_chunks);
    if (dir != 0 && dir != 1) return fail(BP_EINVAL, "direction %d is not 0 or 1", dir);
    if (!grad_out || !grad_in) return fail(BP_EINVAL, "gradient pointer is null");
    const int slot = find_slot(chunk, mb);
    if (slot < 0) return fail(BP_ESTATE, "backward(chunk %d, mb %d) without a stashed forward", chunk, mb);
    auto it = lens.find(mb);
    const int32_t* ln = it == lens.end() ? nullptr : it->second;
    const double unit = (double)T * H * esz;
    const double attn_c = causal ? 0.5 : 1.0;
    int rc;

    // Main stream: the chain of data gradients.  Side stream: weight gradients and column sums,
    // each waiting for the main-stream kernel that produced its input.
    hipStream_t ss = side_stream();
    const bool two = ss != stream;
#define BP_HIP(expr)                                                                    \
    do {                                                                                \
        hipError_t e_ = (expr);                                                         \
        if (e_ != hipSuccess) return fail(BP_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)
    auto hand_over = [&](int k) -> hipError_t {    // side waits for what main has enqueued so far
        if (!two) return hipSuccess;
        hipError_t e = hipEventRecord(ev_ready[k], stream);
        return e != hipSuccess ? e : hipStreamWaitEvent(ss, ev_ready[k], 0);
    };

    if (slots[slot].fwd_pending) {      // the forward that filled the stash ran on the forward stream
        BP_HIP(hipStreamWaitEvent(stream, slots[slot].fwd_done, 0));
        slots[slot].fwd_pending = false;
    }
    if (two && call_done_pending) {
        // the workspaces are shared by all calls: the previous backward's side work must be over
        BP_HIP(hipStreamWaitEvent(stream, ev_misc, 0));
        call_done_pending = false;
        layer_done_pending[0] = layer_done_pending[1] = false;
    }

    // Grouped weight gradients: unless this call completes its group, the four weight-gradient
    // GEMMs of every layer are postponed; the tensors they need (dz, du, dy, dqkv) are then
    // produced straight into a buffer that lives until the group is complete, and the stash stays
    // held.  The call that completes the group multiplies over all waiting micro-batches at once.
    PendGroup& grp = pend[dir][chunk];
    const bool defer = (int)grp.items.size() + 1 < wgrad_group;
    char* qbuf = nullptr;
    if (defer) {
        if (!pend_pool.empty()) {
            qbuf = (char*)pend_pool.back();
            pend_pool.pop_back();
        } else if ((rc = dev_alloc((void**)&qbuf, (size_t)L * q_layer_bytes))) {
            return rc;
        }
    }
    struct PoolGuard {      // hand the buffer back if the call fails half-way
        Stage* st; char*& b;
        ~PoolGuard() { if (b) st->pend_pool.push_back(b); }
    } guard{this, qbuf};

    const void* dz = grad_out;
    if (defer) {            // the caller may reuse grad_out right after this call
        void* keep = qbuf + (size_t)(L - 1) * q_layer_bytes + q_dz;
        BP_HIP(hipMemcpyAsync(keep, grad_out, (size_t)T * H * esz, hipMemcpyDeviceToDevice, stream));
        dz = keep;
    } else if (copy_grad_out) {
        // lanes of bp_run_schedule: the next stage's backward (another lane) rewrites grad_out as soon
        // as this call's main stream is through, so the side stream reads a private copy
        BP_HIP(hipMemcpyAsync(ws_gout, grad_out, (size_t)T * H * esz, hipMemcpyDeviceToDevice, stream));
        dz = ws_gout;
    }
    for (int l = L - 1; l >= 0; --l) {
        const int p = l & 1;
        char* sb = (char*)slots[slot].buf + (size_t)l * s_layer_bytes;
        auto P = [&](int id) { return param(chunk, l, id); };
        auto G = [&](int id) { return grad(dir, chunk, l, id); };
        uint8_t& clean = grad_clean[dir][(size_t)chunk * L + l];
        const int acc = (clean & 1) ? 2 : 1;    // first contribution after a clear overwrites
        char* qb = defer ? qbuf + (size_t)l * q_layer_bytes : nullptr;
        void* dx = l == 0 ? grad_in : defer ? (void*)(qb - q_layer_bytes + q_dz) : ws_dx[l % 3];
        void* big1 = defer ? (void*)(qb + q_du) : ws_big1[p];
        void* big2 = defer ? (void*)(qb + q_dqkv) : ws_big2[p];
        void* h2 = defer ? (void*)(qb + q_dy) : ws_h2[p];
        void *h1 = ws_h1[p], *h5 = ws_h5[p];
        if (two && layer_done_pending[p]) {     // workspaces of this parity still read by the side stream?
            BP_HIP(hipStreamWaitEvent(stream, ev_layer_done[p], 0));
            layer_done_pending[p] = false;
        }
        // column-sum partial regions: db2 | (dgamma2, dbeta2) | dbo | dbqkv | (dgamma1, dbeta1) | db1
        const size_t ch = colsum_chunks(T);
        float* p_b2 = ws_colsum[p];
        float* p_ln2 = p_b2 + ch * H;
        float* p_bo = p_ln2 + ch * 2 * H;
        float* p_bqkv = p_bo + ch * H;
        float* p_ln1 = p_bqkv + ch * 3 * H;
        float* p_b1 = p_ln1 + ch * 2 * H;

        // z = y + g W2 + b2
        BP_HIP(hand_over(0));                                                                               // dz
        if (!defer && (rc = wgrad_one(dir, chunk, l, 0, sb, dz, acc, ss))) return rc;                 // dW2
        {   // du = (dz W2^T) * gelu'(u + b1) with the db1 partials: one kernel when the GEMM can carry it
            GemmArgs bg;
            bg.A = dz; bg.B = P(BP_W2); bg.C = big1; bg.bias = (const float*)P(BP_B1); bg.residual = nullptr;
            bg.M = T; bg.N = F; bg.K = H; bg.lda = H; bg.ldb = H; bg.ldc = F;
            bg.a_t = 0; bg.b_t = 1; bg.accumulate = 0;
            bg.epi = EPI_GELU_BWD; bg.U = sb + s_u; bg.colpart = p_b1;
            if (fuse_gelu && gemm_can_fuse_epilogue(dtype, bg)) {
                prof.tag_gemm(T, F, H, 0, 1, 1, EPI_GELU_BWD);
                Scoped sc(this, BP_K_GEMM, 2.0 * T * (double)F * H, 0);
                BP_LAUNCH(launch_gemm(dtype, bg, stream));
            } else {
                if ((rc = gemm(dz, H, 0, P(BP_W2), H, 1, big1, F, T, F, H, nullptr, nullptr, 0))) return rc;    // dg
                Scoped sc(this, BP_K_GELU_BWD, 0, 3.0 * T * F * esz);
                BP_LAUNCH(launch_gelu_bwd(dtype, T, F, big1, sb + s_u, (const float*)P(BP_B1), big1, nullptr, p_b1,
                                          stream));
            }
        }
        BP_HIP(hand_over(1));                                                                               // du
        if (!defer && (rc = wgrad_one(dir, chunk, l, 1, sb, big1, acc, ss))) return rc;              // dW1
        if ((rc = gemm(big1, F, 0, P(BP_W1), F, 1, h1, H, T, H, F, nullptr, nullptr, 0))) return rc;        // dm
        {   // dy = dz + LN2bwd(dm)
            Scoped sc(this, BP_K_LN_BWD, 0, 4 * unit);
            BP_LAUNCH(launch_ln_bwd_rows(dtype, T, H, h1, sb + s_y, (const float*)(sb + s_mean2),
                                         (const float*)(sb + s_rstd2), (const float*)P(BP_LN2_G), dz, h2, stream));
        }
        // y = x + ctx Wo + bo
        BP_HIP(hand_over(2));                                                                               // dy
        if (!defer && (rc = wgrad_one(dir, chunk, l, 2, sb, h2, acc, ss))) return rc;              // dWo
        if ((rc = gemm(h2, H, 0, P(BP_WO), H, 1, ws_h4, H, T, H, H, nullptr, nullptr, 0))) return rc;       // dctx
        {
            AttnArgs a{B, S, heads, d, causal ? 1 : 0, ln, sb + s_qkv, sb + s_ctx, (float*)(sb + s_lse),
                       ws_h4, big2, ws_delta};
            Scoped sc(this, BP_K_ATTN_BWD, 8.0 * T * S * H * attn_c, 0);
            BP_LAUNCH(launch_attn_bwd(dtype, a, stream));
        }
        // qkv = a Wqkv + bqkv
        BP_HIP(hand_over(3));                                                                               // dqkv
        if (!defer && (rc = wgrad_one(dir, chunk, l, 3, sb, big2, acc, ss))) return rc;              // dWqkv
        if ((rc = gemm(big2, 3 * H, 0, P(BP_WQKV), 3 * H, 1, h5, H, T, H, 3 * H, nullptr, nullptr, 0))) return rc;  // da
        BP_HIP(hand_over(4));                                                                               // da
        {   // every bias and LayerNorm-parameter gradient of the layer in one batched reduction
            ColsumBatch cb;
            cb.n = 6;
            cb.overwrite = (clean & 2) ? 1 : 0;
            cb.jobs[0] = ColsumJob{dz, nullptr, nullptr, nullptr, H, G(BP_B2), nullptr, p_b2};
            cb.jobs[1] = ColsumJob{h1, sb + s_y, (const float*)(sb + s_mean2), (const float*)(sb + s_rstd2), H,
                                   G(BP_LN2_B), G(BP_LN2_G), p_ln2};
            cb.jobs[2] = ColsumJob{h2, nullptr, nullptr, nullptr, H, G(BP_BO), nullptr, p_bo};
            cb.jobs[3] = ColsumJob{big2, nullptr, nullptr, nullptr, 3 * H, G(BP_BQKV), nullptr, p_bqkv};
            cb.jobs[4] = ColsumJob{h5, sb + s_x, (const float*)(sb + s_mean1), (const float*)(sb + s_rstd1), H,
                                   G(BP_LN1_B), G(BP_LN1_G), p_ln1};
            cb.jobs[5] = ColsumJob{nullptr, nullptr, nullptr, nullptr, F, G(BP_B1), nullptr, p_b1};
            Scoped sc(this, BP_K_COLSUM, 0, 0);
            BP_LAUNCH(launch_colsum_batch(dtype, T, cb, ss));
        }
        clean &= defer ? ~2 : 0;
        if (two) {
            BP_HIP(hipEventRecord(ev_layer_done[p], ss));
            layer_done_pending[p] = true;
            if (l == 0 && L > 1) {
                // grad_in may alias grad_out, which the side stream read for the top layer
                const int tp = (L - 1) & 1;
                if (tp != p && layer_done_pending[tp]) {
                    BP_HIP(hipStreamWaitEvent(stream, ev_layer_done[tp], 0));
                    layer_done_pending[tp] = false;
                }
            }
            if (l == 0 && (L == 1 || ((L - 1) & 1) == p)) {
                // same parity as the top layer (or a single layer): its record is the one just made
                BP_HIP(hipStreamWaitEvent(stream, ev_layer_done[p], 0));
                layer_done_pending[p] = false;
            }
        }
        {   // dx = dy + LN1bwd(da)
            Scoped sc(this, BP_K_LN_BWD, 0, 4 * unit);
            BP_LAUNCH(launch_ln_bwd_rows(dtype, T, H, h5, sb + s_x, (const float*)(sb + s_mean1),
                                         (const float*)(sb + s_rstd1), (const float*)P(BP_LN1_G), h2, dx, stream));
        }
        dz = dx;
    }
    slots[slot].live = false;
    if (defer) {
        slots[slot].held = true;
        grp.items.push_back(PendingMb{slot, qbuf});
        qbuf = nullptr;                         // owned by the group now
        note_held();
    } else {
        if ((rc = release_group(grp, ss))) return rc;
        if (two) {
            // the stash may be handed to a new forward only after the side stream has read it
            if (!slots[slot].side_done)
                BP_HIP(hipEventCreateWithFlags(&slots[slot].side_done, hipEventDisableTiming));
            BP_HIP(hipEventRecord(slots[slot].side_done, ss));
            slots[slot].side_pending = true;
        }
    }
    if (two) {
        BP_HIP(hipEventRecord(ev_misc, ss));
        call_done_pending = true;
    }
#undef BP_HIP
    return BP_OK;
}

}  // namespace bp

// ====================================================================== C ABI

using bp::Stage;
using bp::fail;

extern "C" {

int bp_stage_init(bp_stage_t** out, int layers, int hidden, int heads, int seq, int microbatch, int causal) {
    return Stage::create((Stage**)out, layers, hidden, heads, seq, microbatch, causal, nullptr);
}

int bp_stage_init_ex(bp_stage_t** out, int layers, int hidden, int heads, int seq, int microbatch,
                     int causal, const bp_opts* opts) {
    return Stage::create((Stage**)out, layers, hidden, heads, seq, microbatch, causal, opts);
}

size_t bp_stage_stash_bytes(const bp_stage_t* st) {
    if (!st) return 0;
    const Stage* s_ = (const Stage*)st;
    return (size_t)s_->L * s_->s_layer_bytes;
}

int bp_stage_held_bytes(const bp_stage_t* st, size_t* live_stash, size_t* group_stash, size_t* group_grads,
                        size_t* peak_total) {
    if (!st) return fail(BP_EINVAL, "stage handle is null");
    const Stage* s_ = (const Stage*)st;
    size_t h[3];
    s_->held_bytes(h);
    if (live_stash) *live_stash = h[0];
    if (group_stash) *group_stash = h[1];
    if (group_grads) *group_grads = h[2];
    if (peak_total) *peak_total = s_->peak_held_bytes;
    return BP_OK;
}

int bp_stage_reset_peak_bytes(bp_stage_t* st) {
    if (!st) return fail(BP_EINVAL, "stage handle is null");
    Stage* s_ = (Stage*)st;
    s_->peak_held_bytes = 0;
    s_->note_held();
    return BP_OK;
}

int bp_stage_destroy(bp_stage_t* st) {
    delete (Stage*)st;
    return BP_OK;
}

#define BP_ST(st) \
    Stage* s_ = (Stage*)(st); \
    if (!s_) return fail(BP_EINVAL, "stage handle is null")

int bp_stage_set_param(bp_stage_t* st, int chunk, int layer, int id, const float* host, size_t n) {
    BP_ST(st);
    return s_->set_param(chunk, layer, id, host, n);
}
int bp_stage_get_grad(bp_stage_t* st, int chunk, int layer, int id, float* host, size_t n) {
    BP_ST(st);
    return s_->get_grad(chunk, layer, id, host, n);
}
int bp_stage_zero_grad(bp_stage_t* st) {
    BP_ST(st);
    return s_->zero_grad();
}
int bp_stage_wait_forward(bp_stage_t* st) {
    if (!st) return fail(BP_EINVAL, "stage is null");
    return ((Stage*)st)->wait_forward();
}

int bp_stage_merge_directions(bp_stage_t* st) {
    BP_ST(st);
    return s_->merge_directions();
}
int bp_stage_set_seqlens(bp_stage_t* st, int mb, const int32_t* lens) {
    BP_ST(st);
    return s_->set_seqlens(mb, lens);
}
int bp_stage_forward(bp_stage_t* st, int chunk, int mb, const void* act_in, void* act_out) {
    BP_ST(st);
    return s_->forward(chunk, mb, act_in, act_out);
}
int bp_stage_backward(bp_stage_t* st, int chunk, int mb, const void* grad_out, void* grad_in) {
    BP_ST(st);
    return s_->backward(chunk, mb, grad_out, grad_in, 0);
}
int bp_stage_backward_dir(bp_stage_t* st, int chunk, int mb, const void* grad_out, void* grad_in, int dir) {
    BP_ST(st);
    return s_->backward(chunk, mb, grad_out, grad_in, dir);
}

int bp_prof_enable(bp_stage_t* st, int on) {
    BP_ST(st);
    int rc = s_->sync_all();
    if (rc) return rc;
    s_->prof.reset();
    s_->prof.on = on != 0;
    return BP_OK;
}

int bp_prof_get(bp_stage_t* st, int kid, double* ms, long long* launches, double* flops, double* bytes) {
    BP_ST(st);
    if (kid < 0 || kid >= BP_N_KERNEL_IDS) return fail(BP_EINVAL, "kernel id %d out of range", kid);
    if (s_->sync_all()) return BP_EHIP;
    s_->prof.collect();
    if (ms) *ms = s_->prof.ms_total[kid];
    if (launches) *launches = s_->prof.launches[kid];
    if (flops) *flops = s_->prof.flops_total[kid];
    if (bytes) *bytes = s_->prof.bytes_total[kid];
    return BP_OK;
}

int bp_prof_gemm_shapes(bp_stage_t* st) {
    BP_ST(st);
    if (s_->sync_all()) return BP_EHIP;
    s_->prof.collect();
    return (int)s_->prof.shapes.size();
}

int bp_prof_gemm_get(bp_stage_t* st, int index, int* dims, double* total_ms, long long* launches) {
    BP_ST(st);
    if (s_->sync_all()) return BP_EHIP;
    s_->prof.collect();
    if (index < 0 || index >= (int)s_->prof.shapes.size())
        return fail(BP_EINVAL, "shape index %d out of range [0,%zu)", index, s_->prof.shapes.size());
    const auto& sh = s_->prof.shapes[index];
    if (dims) memcpy(dims, sh.dims, sizeof sh.dims);
    if (total_ms) *total_ms = sh.ms;
    if (launches) *launches = sh.launches;
    return BP_OK;
}

const char* bp_last_error(void) { return bp::last_error(); }
const char* bp_version(void) { return "bitpipe-stage-mi355x 0.1 (gfx950)"; }

}  // extern "C"
