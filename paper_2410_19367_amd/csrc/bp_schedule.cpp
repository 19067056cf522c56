// The BitPipe order on the host: V-shaped stage->device map, list-scheduled generation of one
// iteration, validation, a cost-model replay, and the executor that runs an iteration with all
// virtual devices time-sliced on one GPU.
#include <algorithm>
#include <climits>
#include <vector>

#include "bp_host.h"

namespace bp {

// Section 3.2 / 3.3: the down pipeline places stages 0..D-1 on devices 0..D-1 and stages
// D..2D-1 on devices D-1..0; the up pipeline is its mirror image.  With v chunks per device
// (Appendix A) the walk keeps turning round at both ends (0..D-1, D-1..0, 0..D-1, ...), so every
// turn is a local copy; the looping placement of the plain interleaved schedule (the paper's
// "w/o V" ablation) restarts at device 0 instead and has no local copies.
int schedule_vmap(const Layout& L, int dir, int stage, int D) {
    if (D <= 0 || L.v < 1 || stage < 0 || stage >= L.v * D || (dir != 0 && dir != 1)) return -1;
    const int lap = stage / D, pos = stage % D;
    const int down = (L.looping || lap % 2 == 0) ? pos : D - 1 - pos;
    return dir == 0 ? down : D - 1 - down;
}
int schedule_vmap(int dir, int stage, int D) { return schedule_vmap(Layout{}, dir, stage, D); }

// Within each group of D consecutive micro-batches the first half travels down, the second up
// (each pipeline schedules N/2 micro-batches, Section 3.3).
static inline int direction_of(int mb, int D) { return (mb % D) < D / 2 ? 0 : 1; }
// Place of a micro-batch in its own pipeline's injection order (each pipeline runs its micro-batches
// by the 1F1B-Int rule, Section 3.3): the k-th micro-batch of the down pipeline and the k-th of the
// up pipeline rank alike.
static inline int rank_in_pipeline(int mb, int D) { return (mb / D) * (D / 2) + (mb % D) % (D / 2); }

namespace {

struct Timed {
    int start;
    bp_op op;
};

// State of the list scheduler: finish times per (stage, mb), busy-until per device.
struct ListScheduler {
    Layout L;
    int D, N, n_stage, cost_f, cost_b;
    // rule parameters: most chunk stashes per device, most micro-batches in flight, and the stash
    // count below which a device prefers a ready forward to a ready backward (0: never)
    int cap, window, prefer_f_below;
    bool b_lowest_stage_first;               // else: lowest micro-batch first
    std::vector<int> f_done, b_done;        // finish time or INT_MAX while not finished
    std::vector<char> f_started, b_started;
    std::vector<int> busy_until, f_count;
    std::vector<std::vector<int>> b_ends;   // per device: finish times of started backwards
    std::vector<int> admitted;
    std::vector<Timed> out;

    // A stage-activation M_a is v chunk stashes; the caps below are D M_a and (3D-3)/2 M_a.
    ListScheduler(const Layout& L_, int D_, int N_, int cf, int cb, int variant)
        : L(L_), D(D_), N(N_), n_stage(L_.v * D_), cost_f(cf), cost_b(cb),
          cap(variant == BP_SCHED_V_EARLY_FWD ? (D_ > 2 ? ((3 * D_ - 3) * L_.v + 1) / 2 : L_.v * D_) : L_.v * D_),
          window(variant == BP_SCHED_V_EARLY_FWD ? 2 * D_ : D_ + 2),
          prefer_f_below(variant == BP_SCHED_V_EARLY_FWD ? L_.v * D_ : 0),
          b_lowest_stage_first(variant == BP_SCHED_V_EARLY_FWD),
          f_done((size_t)L_.v * D_ * N_, INT_MAX), b_done((size_t)L_.v * D_ * N_, INT_MAX),
          f_started((size_t)L_.v * D_ * N_, 0), b_started((size_t)L_.v * D_ * N_, 0),
          busy_until(D_, 0), f_count(D_, 0), b_ends(D_) {}

    size_t at(int s, int mb) const { return (size_t)mb * n_stage + s; }

    int held(int dev, int t) const {   // stashes alive on dev: forwards started - backwards finished
        int done = 0;
        for (int e : b_ends[dev]) done += e <= t;
        return f_count[dev] - done;
    }
    int in_flight(int t) const {       // admitted micro-batches whose stage-0 backward is not finished
        int n = 0;
        for (int mb : admitted) n += b_done[at(0, mb)] > t;
        return n;
    }

    // Pick what device `dev` starts at time t, or nothing.  Concatenated units: the ready backward
    // of the lowest rank (then lowest stage) unless a backward of lower rank becomes ready in the
    // next slot (a backward holds the device for two slots and would delay it: the device then runs
    // a forward or waits); else the forward of the deepest stage (then lowest rank).  Early
    // forwarding (Appendix B): the forward goes first while the device holds fewer than
    // prefer_f_below stashes, and among backwards the lowest stage wins.
    struct Cand {
        int a, b, c, mb;
        bool operator<(const Cand& o) const {
            if (a != o.a) return a < o.a;
            if (b != o.b) return b < o.b;
            if (c != o.c) return c < o.c;
            return mb < o.mb;
        }
    };
    bool pick(int dev, int t, bp_op* chosen) const {
        bool have_b = false, have_f = false, have_soon = false;
        Cand best_b{}, best_f{}, soon{};
        int b_stage = 0, f_stage = 0;
        const int holding = held(dev, t);
        const bool room = holding < cap;
        const bool may_admit = in_flight(t) < window;
        for (int mb = 0; mb < N; ++mb) {
            const int dir = direction_of(mb, D), rk = rank_in_pipeline(mb, D);
            for (int s = 0; s < n_stage; ++s) {
                if (schedule_vmap(L, dir, s, D) != dev) continue;
                const size_t k = at(s, mb);
                if (!b_started[k]) {
                    const int at_t = std::max(f_done[k], s == n_stage - 1 ? 0 : b_done[at(s + 1, mb)]);
                    const Cand c = b_lowest_stage_first ? Cand{s, rk, dir, mb} : Cand{rk, s, dir, mb};
                    if (at_t <= t) {
                        if (!have_b || c < best_b) { have_b = true; best_b = c; b_stage = s; }
                    } else if (at_t == t + 1 && !b_lowest_stage_first) {
                        if (!have_soon || c < soon) { have_soon = true; soon = c; }
                    }
                }
                if (!f_started[k] && room) {
                    const bool ready = s == 0 ? may_admit : f_done[at(s - 1, mb)] <= t;
                    const Cand c{-s, rk, dir, mb};
                    if (ready && (!have_f || c < best_f)) { have_f = true; best_f = c; f_stage = s; }
                }
            }
        }
        bool take_b = have_b && !(have_f && holding < prefer_f_below);
        if (take_b && have_soon && soon < best_b) {
            take_b = false;                 // a more urgent backward arrives next slot: do not block it
            if (!have_f) return false;
        }
        if (take_b) {
            *chosen = bp_op{1, (int8_t)direction_of(best_b.mb, D), (int16_t)dev, b_stage, best_b.mb};
            return true;
        }
        if (have_f) {
            *chosen = bp_op{0, (int8_t)direction_of(best_f.mb, D), (int16_t)dev, f_stage, best_f.mb};
            return true;
        }
        return false;
    }

    bool run() {
        const size_t total = (size_t)2 * n_stage * N;
        const long horizon = (long)(cost_f + cost_b) * (long)total + 1;
        for (int t = 0; out.size() < total; ++t) {
            if (t > horizon) return false;
            for (int dev = 0; dev < D; ++dev) {
                if (busy_until[dev] > t) continue;
                bp_op op;
                if (!pick(dev, t, &op)) continue;
                const size_t k = at(op.stage, op.mb);
                if (op.kind == 0) {
                    if (op.stage == 0) admitted.push_back(op.mb);
                    f_started[k] = 1;
                    f_done[k] = t + cost_f;
                    f_count[dev] += 1;
                    busy_until[dev] = t + cost_f;
                } else {
                    b_started[k] = 1;
                    b_done[k] = t + cost_b;
                    b_ends[dev].push_back(t + cost_b);
                    busy_until[dev] = t + cost_b;
                }
                out.push_back({t, op});
            }
        }
        return true;
    }
};

}  // namespace

static int check_layout(const Layout& L) {
    if (L.v < 1 || L.v > 64) return fail(BP_EINVAL, "v = %d chunks per device is outside 1..64", L.v);
    return BP_OK;
}

static int schedule_generate(const Layout& L, int D, int N, int variant, bp_op* out, int cap, int* n_out) {
    if (check_layout(L)) return BP_EINVAL;
    if (variant != BP_SCHED_V_CONCAT && variant != BP_SCHED_V_EARLY_FWD)
        return fail(BP_EINVAL, "unknown schedule variant %d", variant);
    if (D < 2 || D % 2) return fail(BP_EINVAL, "D = %d must be even and >= 2", D);
    if (N < D || N % D) return fail(BP_EINVAL, "N = %d must be a positive multiple of D = %d", N, D);
    if (D > 1024 || N > 65536) return fail(BP_EINVAL, "D or N too large");
    const long total = 2L * L.v * D * N;
    if (!out || !n_out || cap < total) return fail(BP_EINVAL, "output array too small (need %ld ops)", total);
    ListScheduler ls(L, D, N, 1, 2, variant);
    if (!ls.run()) return fail(BP_EINVAL, "list scheduler made no progress for D = %d, N = %d", D, N);
    // one GPU runs the devices' ops one after another: order by (start time, device)
    std::stable_sort(ls.out.begin(), ls.out.end(), [](const Timed& a, const Timed& b) {
        return a.start != b.start ? a.start < b.start : a.op.vdev < b.op.vdev;
    });
    for (long i = 0; i < total; ++i) out[i] = ls.out[i].op;
    *n_out = (int)total;
    return BP_OK;
}

int schedule_validate(const Layout& L, const bp_op* order, int n_ops, int D, int N) {
    if (!order) return fail(BP_EINVAL, "order is null");
    if (check_layout(L)) return BP_EINVAL;
    if (D < 2 || D % 2) return fail(BP_EINVAL, "D = %d must be even and >= 2", D);
    if (N < 1) return fail(BP_EINVAL, "N = %d must be positive", N);
    const int n_stage = L.v * D;
    if ((long)n_ops != 2L * n_stage * N)
        return fail(BP_EDEP, "order has %d ops, an iteration needs %ld", n_ops, 2L * n_stage * N);
    std::vector<char> f_seen((size_t)n_stage * N, 0), b_seen((size_t)n_stage * N, 0);
    std::vector<int> mb_dir(N, -1);
    for (int i = 0; i < n_ops; ++i) {
        const bp_op& o = order[i];
        if ((o.kind != 0 && o.kind != 1) || (o.dir != 0 && o.dir != 1))
            return fail(BP_EDEP, "op %d: bad kind or direction", i);
        if (o.stage < 0 || o.stage >= n_stage || o.mb < 0 || o.mb >= N)
            return fail(BP_EDEP, "op %d: stage %d or micro-batch %d out of range", i, o.stage, o.mb);
        if (o.vdev != schedule_vmap(L, o.dir, o.stage, D))
            return fail(BP_EDEP, "op %d: device %d does not match the stage map", i, o.vdev);
        if (mb_dir[o.mb] < 0) mb_dir[o.mb] = o.dir;
        else if (mb_dir[o.mb] != o.dir) return fail(BP_EDEP, "op %d: micro-batch %d changes direction", i, o.mb);
        const size_t k = (size_t)o.mb * n_stage + o.stage;
        if (o.kind == 0) {
            if (f_seen[k]) return fail(BP_EDEP, "op %d: duplicate forward (stage %d, mb %d)", i, o.stage, o.mb);
            if (o.stage > 0 && !f_seen[k - 1])
                return fail(BP_EDEP, "op %d: forward (stage %d, mb %d) before its producer", i, o.stage, o.mb);
            f_seen[k] = 1;
        } else {
            if (b_seen[k]) return fail(BP_EDEP, "op %d: duplicate backward (stage %d, mb %d)", i, o.stage, o.mb);
            if (!f_seen[k]) return fail(BP_EDEP, "op %d: backward (stage %d, mb %d) before its forward", i, o.stage, o.mb);
            if (o.stage < n_stage - 1 && !b_seen[k + 1])
                return fail(BP_EDEP, "op %d: backward (stage %d, mb %d) before its upstream backward", i, o.stage, o.mb);
            b_seen[k] = 1;
        }
    }
    return BP_OK;   // n_ops == 2 * n_stage * N and no duplicates => every op is present
}

static int schedule_simulate(const Layout& L, const bp_op* order, int n_ops, int D, int N, int cost_f, int cost_b,
                             int* makespan, int* idle, int* peak_stash) {
    int rc = schedule_validate(L, order, n_ops, D, N);
    if (rc) return rc;
    if (cost_f <= 0 || cost_b <= 0) return fail(BP_EINVAL, "costs must be positive");
    const int n_stage = L.v * D;
    std::vector<int> f_done((size_t)n_stage * N, 0), b_done((size_t)n_stage * N, 0), busy(D, 0), work(D, 0);
    std::vector<std::vector<std::pair<int, int>>> events(D);   // (time, +1 at F start / -1 at B end)
    int ms = 0;
    for (int i = 0; i < n_ops; ++i) {
        const bp_op& o = order[i];
        const size_t k = (size_t)o.mb * n_stage + o.stage;
        int ready;
        if (o.kind == 0) ready = o.stage == 0 ? 0 : f_done[k - 1];
        else ready = std::max(f_done[k], o.stage == n_stage - 1 ? 0 : b_done[k + 1]);
        const int start = std::max(ready, busy[o.vdev]);
        const int cost = o.kind == 0 ? cost_f : cost_b;
        busy[o.vdev] = start + cost;
        work[o.vdev] += cost;
        if (o.kind == 0) { f_done[k] = start + cost; events[o.vdev].push_back({start, 1}); }
        else { b_done[k] = start + cost; events[o.vdev].push_back({start + cost, -1}); }
        ms = std::max(ms, start + cost);
    }
    if (makespan) *makespan = ms;
    for (int dev = 0; dev < D; ++dev) {
        if (idle) idle[dev] = ms - work[dev];
        if (peak_stash) {
            auto& ev = events[dev];
            std::sort(ev.begin(), ev.end());   // at equal times releases (-1) sort before acquisitions
            int cur = 0, peak = 0;
            for (auto& e : ev) { cur += e.second; peak = std::max(peak, cur); }
            peak_stash[dev] = peak;
        }
    }
    return BP_OK;
}

// Messages of one iteration: every forward hands its output to the next stage and every backward
// its input gradient to the previous one; between different devices that is a P2P message of
// 2 B S H bytes (Appendix C), on the same device (the turns of the zig-zag map) a local copy.
static int schedule_hops(const Layout& L, const bp_op* order, int n_ops, int D, int N, long* p2p, long* local) {
    int rc = schedule_validate(L, order, n_ops, D, N);
    if (rc) return rc;
    const int n_stage = L.v * D;
    long hop = 0, loc = 0;
    for (int i = 0; i < n_ops; ++i) {
        const bp_op& o = order[i];
        const int to = o.kind == 0 ? o.stage + 1 : o.stage - 1;
        if (to < 0 || to >= n_stage) continue;
        (schedule_vmap(L, o.dir, to, D) == o.vdev ? loc : hop) += 1;
    }
    if (p2p) *p2p = hop;
    if (local) *local = loc;
    return BP_OK;
}

// ------------------------------------------------------------------ executor

int Stage::live_slots() const {
    int n = 0;
    for (auto& s : slots) n += s.live;
    return n;
}

// The order on `lanes` lanes: lane l takes the ops of the virtual devices d with d % lanes == l and
// runs them on that lane's view of the object (own streams, workspaces, stash slots; shared
// parameters and gradient buffers).  Every op leaves a completion event on its lane's main stream;
// an op whose producer ran on another lane makes its stream wait for that event (the order respects
// the dependencies, so the event has been recorded by then).  Gradient buffers, weight-gradient
// groups and clear flags belong to one (direction, stage), hence to one device and one lane, so the
// result is the same as with a single lane.  (Enqueueing from one host thread per lane was measured
// too: slower, the runtime serialises the launches.)
int Stage::run_lanes(const Layout& L, const bp_op* order, int n_ops, int D, int N, int lanes, const void* inputs,
                     const void* targets) {
    const int n_stage = L.v * D, last = n_stage - 1;
    const size_t TH = (size_t)T * H, THb = TH * esz;
    const float scale = 1.f / ((float)N * (float)B * (float)S);
    int rc;
    while ((int)views.size() < lanes) {
        Stage* v = nullptr;
        if ((rc = make_view(&v))) return rc;
        views.push_back(v);
    }
    struct ViewGuard {      // a failed run leaves half an iteration's state in the views: drop them
        Stage* s; bool ok = false;
        ~ViewGuard() {
            for (Stage* v : s->views) v->lens.clear();        // not the views' to free
            if (ok) return;
            s->sync_all();
            for (Stage* v : s->views) delete v;
            s->views.clear();
        }
    } guard{this};
#define BP_EV(expr)                                                                     \
    do {                                                                                \
        hipError_t e_ = (expr);                                                         \
        if (e_ != hipSuccess) return fail(BP_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)
    while (sched_ev.size() < (size_t)n_ops) {
        hipEvent_t ev;
        BP_EV(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        sched_ev.push_back(ev);
    }
    if (!ev_fork) BP_EV(hipEventCreateWithFlags(&ev_fork, hipEventDisableTiming));
    // the lanes start after everything enqueued on this object's stream so far
    BP_EV(hipEventRecord(ev_fork, stream));
    std::vector<int> op_of((size_t)2 * n_stage * N, -1);      // (kind, stage, mb) -> position in the order
    for (int i = 0; i < n_ops; ++i)
        op_of[((size_t)order[i].kind * n_stage + order[i].stage) * N + order[i].mb] = i;
    for (int ln = 0; ln < lanes; ++ln) {
        Stage* v = views[ln];
        v->wgrad_group = wgrad_group;
        v->slot_capacity = std::max(v->slot_capacity, n_stage * N);
        // one stream per lane: with four lanes busy a second stream per lane only adds queue traffic
        // (measured: 32.2 ms per cfg4 iteration with side streams, 28.9 ms without)
        v->overlap = false;
        v->copy_grad_out = false;
        v->lens = lens;                                       // key-padding lengths (owned by this object)
        v->grad_clean[0].assign(grad_clean[0].size(), 3);
        v->grad_clean[1].assign(grad_clean[1].size(), 3);
        v->peak_held_bytes = 0;
        BP_EV(hipStreamWaitEvent(v->stream, ev_fork, 0));
    }
    auto lane_of = [&](int dir, int stage) { return schedule_vmap(L, dir, stage, D) % lanes; };
    for (int i = 0; i < n_ops; ++i) {
        const bp_op& o = order[i];
        const int ln = o.vdev % lanes;
        Stage* v = views[ln];
        char* mb_act = (char*)sched_act + (size_t)o.mb * 2 * THb;
        char* mb_grad = (char*)sched_grad + (size_t)o.mb * THb;
        if (o.kind == 0) {
            if (o.stage > 0 && lane_of(o.dir, o.stage - 1) != ln)
                BP_EV(hipStreamWaitEvent(v->stream, sched_ev[op_of[((size_t)0 * n_stage + o.stage - 1) * N + o.mb]], 0));
            const void* in = o.stage == 0 ? (const char*)inputs + (size_t)o.mb * THb
                                          : mb_act + (size_t)((o.stage - 1) & 1) * THb;
            void* out = mb_act + (size_t)(o.stage & 1) * THb;
            if ((rc = v->forward(o.stage, o.mb, in, out))) return rc;
            if (o.stage == last) {
                // loss partials: 1024 floats per micro-batch after the N losses (two lanes may run two losses at once)
                BP_EV(launch_loss(dtype, TH, out, (const char*)targets + (size_t)o.mb * THb, scale, mb_grad,
                                  sched_loss + o.mb, sched_loss + sched_n + (size_t)o.mb * 1024, v->stream));
            }
        } else {
            if (o.stage < last && lane_of(o.dir, o.stage + 1) != ln)
                BP_EV(hipStreamWaitEvent(v->stream, sched_ev[op_of[((size_t)1 * n_stage + o.stage + 1) * N + o.mb]], 0));
            if ((rc = v->backward(o.stage, o.mb, mb_grad, mb_grad, o.dir))) return rc;
        }
        BP_EV(hipEventRecord(sched_ev[i], v->stream));
    }
    // join: weight-gradient groups the iteration left incomplete are flushed on their lanes; this
    // object's streams continue after both streams of every lane, and it takes over the clear flags
    // of the (direction, stage) pairs each lane owns
    size_t peak = 0;
    for (int ln = 0; ln < lanes; ++ln) {
        Stage* v = views[ln];
        if ((rc = v->flush_all())) return rc;
        BP_EV(hipEventRecord(v->ev_ready[0], v->stream));
        BP_EV(hipStreamWaitEvent(stream, v->ev_ready[0], 0));
        BP_EV(hipStreamWaitEvent(side, v->ev_ready[0], 0));
        BP_EV(hipEventRecord(v->ev_ready[1], v->side));
        BP_EV(hipStreamWaitEvent(stream, v->ev_ready[1], 0));
        BP_EV(hipStreamWaitEvent(side, v->ev_ready[1], 0));
        peak += v->peak_held_bytes;
        for (int dir = 0; dir < 2; ++dir)
            for (int st = 0; st < n_stage; ++st) {
                if (lane_of(dir, st) != ln) continue;
                for (int l = 0; l < this->L; ++l)
                    grad_clean[dir][(size_t)st * this->L + l] = v->grad_clean[dir][(size_t)st * this->L + l];
            }
    }
#undef BP_EV
    peak_held_bytes = std::max(peak_held_bytes, peak);        // sum of the lanes' own peaks: an upper bound
    guard.ok = true;
    return BP_OK;
}

int Stage::run_schedule(const Layout& L, const bp_op* order, int n_ops, int D, const void* inputs,
                        const void* targets, float* loss_out) {
    if (!order || !inputs || !targets) return fail(BP_EINVAL, "null argument");
    if (check_layout(L)) return BP_EINVAL;
    if (D < 2 || D % 2) return fail(BP_EINVAL, "D = %d must be even and >= 2", D);
    const int n_stage = L.v * D;
    if (n_chunks != n_stage)
        return fail(BP_EINVAL, "stage object holds %d chunks, the order needs v*D = %d", n_chunks, n_stage);
    if (n_ops <= 0 || n_ops % (2 * n_stage)) return fail(BP_EDEP, "order has %d ops, not a multiple of 2*v*D", n_ops);
    const int N = n_ops / (2 * n_stage);
    int rc = schedule_validate(L, order, n_ops, D, N);
    if (rc) return rc;
    if (live_slots()) return fail(BP_ESTATE, "stashes are live at the start of an iteration");
    // an iteration orders its operations itself: forwards stay on the streams the executor gives them
    int rc_w = wait_forward();
    if (rc_w) return rc_w;
    struct AheadOff {
        Stage* s; bool was;
        ~AheadOff() { s->forward_ahead = was; }
    } ahead_off{this, forward_ahead};
    forward_ahead = false;

    const size_t TH = (size_t)T * H, THb = TH * esz;
    if (sched_n < N) {
        sync_all();
        hipFree(sched_act); hipFree(sched_grad); hipFree(sched_loss);
        sched_act = sched_grad = nullptr; sched_loss = nullptr; sched_n = 0;
        if (hipMalloc(&sched_act, (size_t)N * 2 * THb) != hipSuccess ||
            hipMalloc(&sched_grad, (size_t)N * THb) != hipSuccess ||
            hipMalloc((void**)&sched_loss, ((size_t)N + (size_t)N * 1024) * sizeof(float)) != hipSuccess) {
            (void)hipGetLastError();
            return fail(BP_ENOMEM, "allocating the iteration's hand-off buffers failed");
        }
        sched_n = N;
    }
    // an order may keep every (stage, mb) stashed at once; slots get memory only when used
    if (slot_capacity < n_stage * N) slot_capacity = n_stage * N;

    if ((rc = zero_grad())) return rc;
    // A weight-gradient group that the iteration cannot fill would only be flushed at the end, with
    // nothing left to overlap it: no group larger than the backward calls a (direction, stage) gets.
    struct GroupCap {
        Stage* s; int saved;
        ~GroupCap() { s->wgrad_group = saved; }
    } cap{this, wgrad_group};
    {
        std::vector<int> calls(2 * (size_t)n_stage, 0);
        for (int i = 0; i < n_ops; ++i)
            if (order[i].kind == 1) ++calls[(size_t)order[i].dir * n_stage + order[i].stage];
        for (int c : calls)
            if (c > 0 && c < wgrad_group) wgrad_group = c;
    }
    // Operations of different virtual devices are independent within a time slot, so with the two
    // streams allowed (and no per-launch timing) every virtual device gets a lane of its own; else
    // the ops run one after the other on this object's own lane.
    const int lanes = prof.on || !overlap ? 1 : std::min(D, kMaxLanes);
    if (lanes > 1) {
        if ((rc = run_lanes(L, order, n_ops, D, N, lanes, inputs, targets))) return rc;
    } else {
        const int last = n_stage - 1;
        const float scale = 1.f / ((float)N * (float)B * (float)S);
        for (int i = 0; i < n_ops; ++i) {
            const bp_op& o = order[i];
            // stage s writes hand-off buffer s%2 of its micro-batch and reads the other one: the
            // P2P message between devices, or the local copy at the V turn
            char* mb_act = (char*)sched_act + (size_t)o.mb * 2 * THb;
            char* mb_grad = (char*)sched_grad + (size_t)o.mb * THb;
            if (o.kind == 0) {
                const void* in = o.stage == 0 ? (const char*)inputs + (size_t)o.mb * THb
                                              : mb_act + (size_t)((o.stage - 1) & 1) * THb;
                void* out = mb_act + (size_t)(o.stage & 1) * THb;
                if ((rc = forward(o.stage, o.mb, in, out))) return rc;
                if (o.stage == last) {
                    struct Guard { Stage* s; Guard(Stage* st) : s(st) { s->prof.begin(s, BP_K_OTHER, 0, 0); } ~Guard() { s->prof.end(s); } } g(this);
                    hipError_t e = launch_loss(dtype, TH, out, (const char*)targets + (size_t)o.mb * THb, scale,
                                               mb_grad, sched_loss + o.mb, sched_loss + sched_n + (size_t)o.mb * 1024, stream);
                    if (e != hipSuccess) return fail(BP_EHIP, "loss kernel: %s", hipGetErrorString(e));
                }
            } else {
                if ((rc = backward(o.stage, o.mb, mb_grad, mb_grad, o.dir))) return rc;
            }
        }
    }
    if ((rc = merge_directions())) return rc;
    std::vector<float> host_loss(N);
    hipError_t e = hipMemcpyAsync(host_loss.data(), sched_loss, N * sizeof(float), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail(BP_EHIP, "end of iteration: %s", hipGetErrorString(e));
    if ((rc = sync_all())) return rc;
    if (loss_out) {
        double s = 0.0;
        for (int m = 0; m < N; ++m) s += host_loss[m];
        *loss_out = (float)s;
    }
    return BP_OK;
}

}  // namespace bp

extern "C" {

static bp::Layout layout_of(const bp_layout* l) {
    bp::Layout L;
    if (l) { L.v = l->v; L.looping = l->looping != 0; }
    return L;
}

int bp_schedule_vmap(int dir, int stage, int D) { return bp::schedule_vmap(dir, stage, D); }
int bp_schedule_vmap_ex(const bp_layout* l, int dir, int stage, int D) {
    return bp::schedule_vmap(layout_of(l), dir, stage, D);
}

int bp_schedule_generate(int D, int N, int variant, bp_op* out, int cap, int* n_out) {
    return bp::schedule_generate(bp::Layout{}, D, N, variant, out, cap, n_out);
}
int bp_schedule_generate_ex(const bp_layout* l, int D, int N, int variant, bp_op* out, int cap, int* n_out) {
    return bp::schedule_generate(layout_of(l), D, N, variant, out, cap, n_out);
}

int bp_schedule_validate(const bp_op* order, int n_ops, int D, int N) {
    return bp::schedule_validate(bp::Layout{}, order, n_ops, D, N);
}
int bp_schedule_validate_ex(const bp_layout* l, const bp_op* order, int n_ops, int D, int N) {
    return bp::schedule_validate(layout_of(l), order, n_ops, D, N);
}

int bp_schedule_simulate(const bp_op* order, int n_ops, int D, int N, int cost_f, int cost_b,
                         int* makespan, int* idle, int* peak_stash) {
    return bp::schedule_simulate(bp::Layout{}, order, n_ops, D, N, cost_f, cost_b, makespan, idle, peak_stash);
}
int bp_schedule_simulate_ex(const bp_layout* l, const bp_op* order, int n_ops, int D, int N, int cost_f,
                            int cost_b, int* makespan, int* idle, int* peak_stash) {
    return bp::schedule_simulate(layout_of(l), order, n_ops, D, N, cost_f, cost_b, makespan, idle, peak_stash);
}

int bp_schedule_hops(const bp_layout* l, const bp_op* order, int n_ops, int D, int N, long* p2p, long* local) {
    return bp::schedule_hops(layout_of(l), order, n_ops, D, N, p2p, local);
}

int bp_run_schedule(bp_stage_t* st, const bp_op* order, int n_ops, int D, const void* inputs,
                    const void* targets, float* loss_out) {
    if (!st) return bp::fail(BP_EINVAL, "stage handle is null");
    return ((bp::Stage*)st)->run_schedule(bp::Layout{}, order, n_ops, D, inputs, targets, loss_out);
}
int bp_run_schedule_ex(bp_stage_t* st, const bp_layout* l, const bp_op* order, int n_ops, int D,
                       const void* inputs, const void* targets, float* loss_out) {
    if (!st) return bp::fail(BP_EINVAL, "stage handle is null");
    return ((bp::Stage*)st)->run_schedule(layout_of(l), order, n_ops, D, inputs, targets, loss_out);
}

}  // extern "C"
