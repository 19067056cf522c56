"""CPU oracle for the BitPipe V-shaped bidirectional order (pure Python).

TEST INFRASTRUCTURE ONLY; shares nothing with the library's own generator/validator.

From the paper (arXiv 2410.19367):
  * V-shaped map (Section 3.2): a pipeline has 2D stages on D devices; stages 1..D sit on
    devices P1..PD and stages D+1..2D on PD..P1, so the hop D -> D+1 is a local copy.
  * Two such pipelines in opposite directions are merged (Section 3.3): the "down" pipeline
    enters at P1, the "up" pipeline is the mirror image and enters at PD; each schedules N/2
    micro-batches; for even D no two ops collide on a device.
  * With t_b = 2 t_f the basic unit (N = D) has bubble ratio (D-2)/(3N+D-2), made of (D-2)/2
    forward bubbles and (D-2)/4 backward bubbles per device (Section 3.3, Table 2), and holds
    between (D+3)/2 and D stage-activations M_a per device (Table 2).
  * N = K*D micro-batches: K basic units concatenated; the next unit's first forwards fill the
    previous unit's tail bubbles (Section 3.5).
The figures that draw the slot-by-slot order are not available, so the order is rebuilt by
deterministic list scheduling under the unit-cost model (a chunk forward costs 1, a chunk
backward 2; a stage-activation M_a is two chunk stashes).  Each pipeline runs its N/2 micro-batches
by the 1F1B-Int rule (Section 3.3), so what ranks a micro-batch is its place in its own pipeline's
injection order (the k-th micro-batch of the down pipeline and the k-th of the up pipeline rank
alike), not its global index.  A free device runs the ready backward of the lowest rank, otherwise
the ready forward of the highest stage (lowest rank first); it does not start a backward when one
of lower rank becomes ready in the next slot (a backward holds the device for two slots, so
starting it would delay the more urgent one): it then runs a forward, or waits one slot.  A device
never holds more than 2D chunk stashes, and a micro-batch is admitted only while fewer than D + 2
are in flight.  For the basic unit N = D this reproduces the paper's closed forms (makespan 8D - 4
chunk slots = 3N + D - 2 device-forwards, idle 2(D-2) per device) for every even D tested, 4 to 16;
for N = K*D it comes within a few per cent of (D-2)/(3N+D-2) but does not reach it exactly
(parity unpinned for N > D beyond what the tests state).
  * Early forwarding (Appendix B, Eq. 1-2): for N > D, forwards of later micro-batches are run
    ahead of time so that the bubbles between concatenated units disappear; the bubble ratio drops
    to (D-2)/(4N+D-2) (idle (D-2)/4 (t_f + t_b) per device) at a peak of (3D-3)/2 M_a.  Rebuilt
    here as a second list-scheduling rule: a device that holds fewer than 2D chunk stashes prefers
    a ready forward (deepest stage first), one that holds 2D or more prefers a ready backward
    (lowest stage first, i.e. the one closest to releasing its micro-batch); never more than
    3D-3 chunk stashes per device, at most 2D micro-batches in flight.  At D = 4 and N = 2D..6D
    this gives exactly makespan 6N + 3, idle 3 per device and peak 9 = 3D-3 chunk stashes: the
    paper's closed forms.  For D > 4 it does not reach them in general (parity unpinned).
"""
from __future__ import annotations

from collections import namedtuple

Op = namedtuple("Op", "kind direction vdev stage mb")   # kind 'F'|'B'; direction 0 down, 1 up
Slot = namedtuple("Slot", "start end op")


def vmap_down(stage, D, v=2, looping=False):
    """Device (0-based) of 0-based stage s in the down pipeline of v*D stages.  Zig-zag (the V
    shape for v = 2; Appendix A for more chunks per device): laps 0, 2, ... run 0..D-1 and laps
    1, 3, ... run D-1..0, so consecutive laps meet on one device.  Looping (the interleaved
    placement the paper's "w/o V" ablation falls back to): every lap runs 0..D-1."""
    lap, pos = divmod(stage, D)
    if not 0 <= lap < v:
        raise ValueError("stage out of range")
    return pos if looping or lap % 2 == 0 else D - 1 - pos


def vmap(direction, stage, D, v=2, looping=False):
    """Device of a stage in the down (0) or up (1, mirrored) pipeline."""
    d = vmap_down(stage, D, v, looping)
    return d if direction == 0 else D - 1 - d


def direction_of(mb, D):
    """Within each basic unit of D micro-batches the first D/2 go down, the rest up."""
    return 0 if (mb % D) < D // 2 else 1


def rank_in_pipeline(mb, D):
    """Place of a micro-batch in its own pipeline's injection order (both pipelines count alike):
    units of D micro-batches in sequence, inside a unit the first D/2 go down and the last D/2 up."""
    unit, r = divmod(mb, D)
    return unit * (D // 2) + r % (D // 2)


def generate_timeline(D, N, cost_f=1, cost_b=2, early_forward=False, v=2, looping=False):
    """List-schedule one iteration.  Returns per-device lists of Slot(start, end, op).

    Time advances in unit steps; at each step the devices are visited in index order and a free
    device starts at most one op whose inputs finished at or before that step.  A forward needs
    a free stash slot on its device (cap 2D chunk stashes = D * M_a; a slot is given back when
    the backward finishes).  A micro-batch is admitted (stage-0 forward) only while fewer than
    D + 2 admitted micro-batches still await their stage-0 backward: that lets the next basic
    unit's first forwards fill the tail bubbles of the previous one without flooding the
    stashes.  Priorities: see the module header.  early_forward selects the Appendix-B rule
    described there instead.
    v, looping: other stage placements (see vmap_down); a stage-activation M_a is then v chunk
    stashes and the stash caps scale with it.  Raises RuntimeError if the greedy order stalls."""
    if D < 2 or D % 2 or N < D or N % D:
        raise ValueError("need even D >= 2 and N a positive multiple of D")
    if v < 1:
        raise ValueError("need at least one chunk per device")
    n_stage = v * D
    if early_forward:
        cap = -(-(3 * D - 3) * v // 2) if D > 2 else v * D      # (3D-3)/2 M_a, rounded up
        window = 2 * D
        prefer_f_below = v * D
    else:
        cap = v * D                         # D M_a
        window = D + 2
        prefer_f_below = 0                  # always backwards first
    done_f, done_b = {}, {}             # (stage, mb) -> finish time
    free_at = [0] * D
    lanes = [[] for _ in range(D)]
    started = set()
    admitted = []
    total = 2 * n_stage * N
    horizon = (cost_f + cost_b) * total + 1     # every op run alone, one after another
    never = 1 << 60
    t = 0
    while len(started) < total:
        if t > horizon:
            raise RuntimeError("list scheduler made no progress")
        for dev in range(D):
            if free_at[dev] > t:
                continue
            held = sum(1 for sl in lanes[dev] if sl.op.kind == "F") - \
                sum(1 for sl in lanes[dev] if sl.op.kind == "B" and sl.end <= t)
            in_flight = sum(1 for mb in admitted if done_b.get((0, mb), never) > t)
            ready_b, ready_f, soon_b = [], [], []
            for mb in range(N):
                dr = direction_of(mb, D)
                rk = rank_in_pipeline(mb, D)
                for s in range(n_stage):
                    if vmap(dr, s, D, v, looping) != dev:
                        continue
                    if ("B", s, mb) not in started:
                        at = max(done_f.get((s, mb), never),
                                 0 if s == n_stage - 1 else done_b.get((s + 1, mb), never))
                        if at <= t:
                            ready_b.append((rk, s, dr, mb))
                        elif at == t + 1:
                            soon_b.append((rk, s, dr, mb))
                    if ("F", s, mb) not in started and held < cap:
                        if s == 0:
                            if in_flight < window:
                                ready_f.append((0, rk, dr, mb))
                        elif done_f.get((s - 1, mb), never) <= t:
                            ready_f.append((-s, rk, dr, mb))
            pick_b = None
            if ready_b and not (ready_f and held < prefer_f_below):
                if early_forward:       # lowest stage first, then lowest rank
                    pick_b = min(ready_b, key=lambda c: (c[1], c[0], c[2]))
                else:                   # lowest rank first, then lowest stage
                    pick_b = min(ready_b)
                    if soon_b and min(soon_b) < pick_b:
                        pick_b = None   # a more urgent backward arrives next slot: do not block it
                        if not ready_f:
                            continue
            if pick_b is not None:
                rk, s, dr, mb = pick_b
                started.add(("B", s, mb))
                done_b[(s, mb)] = t + cost_b
                free_at[dev] = t + cost_b
                lanes[dev].append(Slot(t, t + cost_b, Op("B", dr, dev, s, mb)))
            elif ready_f:
                ns, rk, dr, mb = min(ready_f)
                s = -ns
                if s == 0:
                    admitted.append(mb)
                started.add(("F", s, mb))
                done_f[(s, mb)] = t + cost_f
                free_at[dev] = t + cost_f
                lanes[dev].append(Slot(t, t + cost_f, Op("F", dr, dev, s, mb)))
        t += 1
    return lanes


def serialise(lanes):
    """One GPU runs the devices' ops one after another: sort by (start time, device)."""
    slots = [sl for lane in lanes for sl in lane]
    slots.sort(key=lambda sl: (sl.start, sl.op.vdev))
    return [sl.op for sl in slots]


def generate(D, N, early_forward=False, v=2, looping=False):
    return serialise(generate_timeline(D, N, early_forward=early_forward, v=v, looping=looping))


def makespan(lanes):
    return max(sl.end for lane in lanes for sl in lane)


def idle_per_device(lanes):
    ms = makespan(lanes)
    return [ms - sum(sl.end - sl.start for sl in lane) for lane in lanes]


def peak_stash(lanes):
    """Max number of simultaneously held chunk stashes per device (F start .. B end)."""
    peaks = []
    for lane in lanes:
        ev = []
        for sl in lane:
            if sl.op.kind == "F":
                ev.append((sl.start, 1))
            else:
                ev.append((sl.end, -1))
        ev.sort(key=lambda e: (e[0], e[1]))
        cur = peak = 0
        for _, dlt in ev:
            cur += dlt
            peak = max(peak, cur)
        peaks.append(peak)
    return peaks


def conflicts(lanes):
    """Number of overlapping slot pairs on any device (must be 0)."""
    bad = 0
    for lane in lanes:
        s = sorted(lane, key=lambda sl: sl.start)
        for a, b in zip(s, s[1:]):
            if b.start < a.end:
                bad += 1
    return bad


def validate(order, D, N, v=2, looping=False):
    """Check a serial order: every (stage, mb) has exactly one F and one B, each op's inputs
    precede it, the device matches the V map, a micro-batch keeps one direction.
    Returns None if valid, else a message naming the first violation."""
    n_stage = v * D
    seen_f, seen_b, mb_dir = set(), set(), {}
    for i, op in enumerate(order):
        if op.kind not in ("F", "B") or op.direction not in (0, 1):
            return f"op {i}: bad kind/direction"
        if not (0 <= op.stage < n_stage and 0 <= op.mb < N):
            return f"op {i}: stage/mb out of range"
        if op.vdev != vmap(op.direction, op.stage, D, v, looping):
            return f"op {i}: device does not match the stage map"
        if mb_dir.setdefault(op.mb, op.direction) != op.direction:
            return f"op {i}: micro-batch changes direction"
        key = (op.stage, op.mb)
        if op.kind == "F":
            if key in seen_f:
                return f"op {i}: duplicate forward"
            if op.stage > 0 and (op.stage - 1, op.mb) not in seen_f:
                return f"op {i}: forward before its producer"
            seen_f.add(key)
        else:
            if key in seen_b:
                return f"op {i}: duplicate backward"
            if key not in seen_f:
                return f"op {i}: backward before its forward"
            if op.stage < n_stage - 1 and (op.stage + 1, op.mb) not in seen_b:
                return f"op {i}: backward before its upstream backward"
            seen_b.add(key)
    if len(seen_f) != n_stage * N or len(seen_b) != n_stage * N:
        return "missing ops"
    return None


def cross_device_hops(order, D, v=2, looping=False):
    """(cross-device hops, local copies) of the forward passes of one micro-batch's pipeline."""
    hops = local = 0
    mb0 = order[0].mb
    dr = [op.direction for op in order if op.mb == mb0][0]
    for s in range(1, v * D):
        if vmap(dr, s, D, v, looping) == vmap(dr, s - 1, D, v, looping):
            local += 1
        else:
            hops += 1
    return hops, local


def messages(order, D, v=2, looping=False):
    """(P2P messages, local copies) of a whole iteration: each forward hands its output to the
    next stage, each backward its input gradient to the previous one (Appendix C counts both)."""
    p2p = local = 0
    for op in order:
        to = op.stage + 1 if op.kind == "F" else op.stage - 1
        if 0 <= to < v * D:
            if vmap(op.direction, to, D, v, looping) == op.vdev:
                local += 1
            else:
                p2p += 1
    return p2p, local
