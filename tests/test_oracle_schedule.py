"""Pins for the schedule oracle: the V map, direction split, conflict-freeness, the closed
forms the paper prints for the basic unit, dependency validity, and hop counts."""
import random
from fractions import Fraction

import pytest

from oracle import schedule_oracle as so


def _golden_rows():
    import os
    p = os.path.join(os.path.dirname(__file__), "golden", "paper_bitpipe_closed_forms.txt")
    rows = []
    for line in open(p):
        line = line.strip()
        if not line or line.startswith("#") or line.startswith("EF"):
            continue
        rows.append([float(v) for v in line.split()])
    return rows


def test_vmap_matches_section_3_2_example():
    # D = 2: stages 1..2 on P1..P2, stages 3..4 on P2..P1
    assert [so.vmap(0, s, 2) for s in range(4)] == [0, 1, 1, 0]
    # D = 4 down: stages 1..4 -> P1..P4, 5..8 -> P4..P1; up is the mirror image
    assert [so.vmap(0, s, 4) for s in range(8)] == [0, 1, 2, 3, 3, 2, 1, 0]
    assert [so.vmap(1, s, 4) for s in range(8)] == [3, 2, 1, 0, 0, 1, 2, 3]


@pytest.mark.parametrize("D", [2, 4, 6, 8])
def test_vmap_properties(D):
    for dr in (0, 1):
        devs = [so.vmap(dr, s, D) for s in range(2 * D)]
        # every device holds exactly two chunks per direction; the turn is a local copy
        assert sorted(devs) == sorted(list(range(D)) * 2)
        assert devs[D - 1] == devs[D]
        # every other hop goes to a neighbouring device
        for s in range(1, 2 * D):
            if s != D:
                assert abs(devs[s] - devs[s - 1]) == 1
    # the two replicas of a stage sit on devices d and D-1-d
    for s in range(2 * D):
        assert so.vmap(0, s, D) + so.vmap(1, s, D) == D - 1


@pytest.mark.parametrize("D,N", [(2, 2), (4, 4), (4, 8), (6, 6), (4, 16)])
def test_direction_split_half_and_half(D, N):
    dirs = [so.direction_of(m, D) for m in range(N)]
    assert dirs.count(0) == dirs.count(1) == N // 2
    for u in range(N // D):
        assert dirs[u * D:u * D + D // 2] == [0] * (D // 2)
        assert dirs[u * D + D // 2:(u + 1) * D] == [1] * (D // 2)


@pytest.mark.parametrize("D,N", [(2, 2), (2, 4), (4, 4), (4, 8), (4, 16), (6, 6), (6, 12), (8, 8)])
def test_generated_order_is_valid_and_conflict_free(D, N):
    lanes = so.generate_timeline(D, N)
    assert so.conflicts(lanes) == 0
    order = so.serialise(lanes)
    assert len(order) == 2 * 2 * D * N
    assert so.validate(order, D, N) is None
    # exactly one F and one B per (stage, mb)
    assert len({(o.kind, o.stage, o.mb) for o in order}) == len(order)
    # never more than 2D chunk stashes (= D stage-activations) on a device
    assert max(so.peak_stash(lanes)) <= 2 * D
    # every device does the same amount of work: 2 chunks/direction * N/2 mbs * 2 directions
    for lane in lanes:
        assert sum(sl.end - sl.start for sl in lane) == 3 * 2 * N


@pytest.mark.parametrize("row", _golden_rows())
def test_basic_unit_closed_forms(row):
    """Section 3.3 / Table 2 for the basic unit N = D at D = 4, 6, 8, 10, 12, 16, read from the golden
    fixture (the paper's formulas evaluated at those D)."""
    D, N, fb, bb, num, den, lo, hi = row
    D, N = int(D), int(N)
    lanes = so.generate_timeline(D, N)
    assert so.conflicts(lanes) == 0 and so.validate(so.serialise(lanes), D, N) is None
    ms = so.makespan(lanes)
    # one device-forward = 2 chunk units; total time 3N + D - 2 device-forwards
    assert ms == 2 * int(den) == 8 * D - 4
    idle = so.idle_per_device(lanes)
    assert all(Fraction(i, ms) == Fraction(int(num), int(den)) for i in idle)
    # idle = (D-2)/2 forward bubbles + (D-2)/4 backward bubbles, of 2 and 4 chunk units each
    assert all(i == int(fb * 2 + bb * 4) == 2 * (D - 2) for i in idle)
    # activations between (D+3)/2 and D stage-activations M_a (= 2 chunk stashes each): the busiest
    # device holds exactly D M_a, none holds less than the lower end of the paper's range
    peaks = so.peak_stash(lanes)
    assert max(peaks) == int(hi * 2) == 2 * D
    assert min(peaks) >= int(lo * 2) == D + 3
    assert peaks == peaks[::-1]                       # the two pipelines mirror each other
    if D == 4:
        assert peaks == [7, 8, 8, 7]                  # here the lower end is reached too


def test_rank_not_global_index_orders_the_backwards():
    """Planted mistake: ranking backwards by the global micro-batch index (every down micro-batch
    before every up one) instead of by the place in the own pipeline misses the closed form from
    D = 6 on; the pins above would catch it."""
    real = so.rank_in_pipeline
    try:
        so.rank_in_pipeline = lambda mb, D: mb
        assert so.makespan(so.generate_timeline(6, 6)) > 8 * 6 - 4
        assert so.makespan(so.generate_timeline(8, 8)) > 8 * 8 - 4
    finally:
        so.rank_in_pipeline = real
    assert so.makespan(so.generate_timeline(6, 6)) == 44


def test_concatenation_fills_tail_bubbles_D4():
    """Section 3.5: N = 2D must beat two basic units back to back (56) and cannot beat the
    closed form 2*(3N + D - 2) = 52; the list-scheduled order lands at 53.  For N = K D the order
    stays within 7 % of the closed form (D-2)/(3N+D-2) at the sizes below but does not reach it."""
    ms = so.makespan(so.generate_timeline(4, 8))
    assert 52 <= ms < 56
    assert ms == 53
    for D, N in ((4, 12), (4, 16), (6, 12), (8, 16), (8, 24)):
        closed = 6 * N + 2 * D - 4
        got = so.makespan(so.generate_timeline(D, N))
        assert closed <= got <= 1.07 * closed, (D, N, got, closed)
        assert got < (N // D) * (8 * D - 4)            # better than units back to back


def _golden_early_forward_rows():
    import os
    p = os.path.join(os.path.dirname(__file__), "golden", "paper_bitpipe_closed_forms.txt")
    return [[float(v) for v in line.split()[1:]] for line in open(p) if line.startswith("EF")]


@pytest.mark.parametrize("row", _golden_early_forward_rows())
def test_early_forwarding_closed_forms_D4(row):
    """Appendix B, Eq. 1-2 at D = 4 from the golden fixture: idle (D-2)/4 (t_f + t_b) per device
    with t_f = 2, t_b = 4 chunk units, bubble ratio (D-2)/(4N+D-2), peak (3D-3)/2 M_a = 3D-3
    chunk stashes; and the order is a valid, conflict-free BitPipe iteration."""
    D, N, num, den, idle_df, peak_ma = row
    D, N = int(D), int(N)
    lanes = so.generate_timeline(D, N, early_forward=True)
    assert so.conflicts(lanes) == 0
    assert so.validate(so.serialise(lanes), D, N) is None
    ms = so.makespan(lanes)
    idle = so.idle_per_device(lanes)
    assert all(i == int(idle_df * 2) == 3 for i in idle)
    assert ms == 6 * N + 3                                  # ideal N (t_f + t_b) plus the bubbles
    assert all(Fraction(i, ms) == Fraction(int(num), int(den)) for i in idle)
    assert max(so.peak_stash(lanes)) == int(peak_ma * 2) == 3 * D - 3
    # fewer bubbles than direct concatenation, whose closed form is 2 (3N + D - 2)
    assert ms < 2 * (3 * N + D - 2) <= so.makespan(so.generate_timeline(D, N))


@pytest.mark.parametrize("D,N", [(2, 4), (4, 4), (6, 12), (8, 16), (8, 32)])
def test_early_forwarding_orders_are_valid_for_other_sizes(D, N):
    """Beyond the pinned sizes the rule still has to give a complete, dependency-respecting,
    conflict-free order within its stash cap (the closed forms are not claimed there)."""
    lanes = so.generate_timeline(D, N, early_forward=True)
    assert so.conflicts(lanes) == 0
    assert so.validate(so.serialise(lanes), D, N) is None
    assert max(so.peak_stash(lanes)) <= max(3 * D - 3, 2 * D if D == 2 else 0)


def test_d2_has_no_bubbles():
    # (D-2)/(3N+D-2) = 0 at D = 2
    for N in (2, 4, 8):
        lanes = so.generate_timeline(2, N)
        assert so.idle_per_device(lanes) == [0, 0]


def test_hops_per_pass():
    # one pass over 2D stages: 2D-2 cross-device hops and one local copy (Section 3.2)
    for D in (2, 4, 8):
        hops, local = so.cross_device_hops(so.generate(D, D), D)
        assert (hops, local) == (2 * D - 2, 1)
    # whole iteration: forward and backward passes of N micro-batches -> 2N(2D-2) messages
    D, N = 4, 8
    order = so.generate(D, N)
    msgs = 0
    for o in order:
        nxt = o.stage + 1 if o.kind == "F" else o.stage - 1
        if 0 <= nxt < 2 * D and so.vmap(o.direction, nxt, D) != o.vdev:
            msgs += 1
    assert msgs == 2 * N * (2 * D - 2)


def test_validator_rejects_planted_mistakes():
    D, N = 4, 4
    good = so.generate(D, N)
    assert so.validate(good, D, N) is None
    # drop an op
    assert so.validate(good[:-1], D, N) is not None
    # duplicate an op
    assert so.validate(good + [good[0]], D, N) is not None
    # swap a backward in front of its forward
    i = next(k for k, o in enumerate(good) if o.kind == "B")
    j = next(k for k, o in enumerate(good) if o.kind == "F" and (o.stage, o.mb) == (good[i].stage, good[i].mb))
    bad = list(good)
    bad[i], bad[j] = bad[j], bad[i]
    assert so.validate(bad, D, N) is not None
    # wrong device
    bad = list(good)
    bad[3] = bad[3]._replace(vdev=(bad[3].vdev + 1) % D)
    assert so.validate(bad, D, N) is not None
    # forward of stage s+1 before stage s
    bad = [o for o in good]
    k1 = next(k for k, o in enumerate(bad) if o.kind == "F" and o.stage == 1 and o.mb == 0)
    k0 = next(k for k, o in enumerate(bad) if o.kind == "F" and o.stage == 0 and o.mb == 0)
    bad[k0], bad[k1] = bad[k1], bad[k0]
    assert so.validate(bad, D, N) is not None


def test_random_topological_orders_validate():
    """Any linear extension of the dependency DAG is a valid order for the executor."""
    D, N = 4, 4
    base = so.generate(D, N)
    rng = random.Random(0)
    for _ in range(5):
        pending = list(base)
        out, seen = [], set()
        while pending:
            ready = []
            for o in pending:
                if o.kind == "F":
                    ok = o.stage == 0 or ("F", o.stage - 1, o.mb) in seen
                else:
                    ok = ("F", o.stage, o.mb) in seen and (
                        o.stage == 2 * D - 1 or ("B", o.stage + 1, o.mb) in seen)
                if ok:
                    ready.append(o)
            o = rng.choice(ready)
            pending.remove(o)
            seen.add((o.kind, o.stage, o.mb))
            out.append(o)
        assert so.validate(out, D, N) is None


def test_bad_arguments():
    for D, N in [(3, 3), (4, 6), (0, 4), (4, 2)]:
        with pytest.raises(ValueError):
            so.generate_timeline(D, N)


def _fits_in(D, N, T):
    """Time-indexed integer program: can one iteration of the V-mapped bidirectional pipeline
    (chunk forward 1 slot, chunk backward 2 slots, one op per device at a time, dependencies along
    each micro-batch's forward and backward chain) finish within T slots?  Independent of the
    list scheduler: only the V map and the direction split are shared with it."""
    import numpy as np
    from scipy.optimize import Bounds, LinearConstraint, milp
    from scipy.sparse import lil_matrix
    n_stage = 2 * D
    ops = []                                        # (kind, stage, mb, device, duration, earliest, latest start)
    for mb in range(N):
        dr = so.direction_of(mb, D)
        for s in range(n_stage):
            dev = so.vmap(dr, s, D)
            ops.append(("F", s, mb, dev, 1, s, T - ((n_stage - s) + 2 * n_stage)))
            ops.append(("B", s, mb, dev, 2, n_stage + 2 * (n_stage - 1 - s), T - 2 * (s + 1)))
    var = {}
    for o, (_, _, _, _, _, lo_t, hi_t) in enumerate(ops):
        if hi_t < lo_t:
            return False                            # not even one micro-batch's chain fits
        for t in range(lo_t, hi_t + 1):
            var[(o, t)] = len(var)
    index = {(k, s, mb): o for o, (k, s, mb, *_rest) in enumerate(ops)}
    rows, lo, hi = [], [], []

    def starts(o):
        return range(ops[o][5], ops[o][6] + 1)

    for o in range(len(ops)):                       # every op starts exactly once
        rows.append({var[(o, t)]: 1.0 for t in starts(o)}); lo.append(1); hi.append(1)

    def after(first, second):                       # start(second) >= start(first) + duration(first)
        row = {var[(second, t)]: float(t) for t in starts(second)}
        for t in starts(first):
            row[var[(first, t)]] = row.get(var[(first, t)], 0.0) - t
        rows.append(row); lo.append(ops[first][4]); hi.append(np.inf)

    for mb in range(N):
        for s in range(n_stage):
            if s > 0:
                after(index[("F", s - 1, mb)], index[("F", s, mb)])
            if s < n_stage - 1:
                after(index[("B", s + 1, mb)], index[("B", s, mb)])
            else:
                after(index[("F", s, mb)], index[("B", s, mb)])
    for dev in range(D):                            # a device runs one op at a time
        for tau in range(T):
            row = {}
            for o, (_, _, _, d2, dur, _, _) in enumerate(ops):
                if d2 == dev:
                    for t in starts(o):
                        if t <= tau < t + dur:
                            row[var[(o, t)]] = 1.0
            rows.append(row); lo.append(0); hi.append(1)
    A = lil_matrix((len(rows), len(var)))
    for i, row in enumerate(rows):
        for v, c in row.items():
            A[i, v] = c
    res = milp(np.zeros(len(var)), constraints=LinearConstraint(A.tocsr(), lo, hi),
               integrality=np.ones(len(var)), bounds=Bounds(0, 1), options={"time_limit": 60})
    assert res.status in (0, 2), res.message       # solved, or proven infeasible
    return res.status == 0


@pytest.mark.parametrize("N,closed_form", [(4, 28), (8, 51), (12, 75)])
def test_closed_forms_are_lower_bounds_at_D4(N, closed_form):
    """No order at all (with any amount of stash memory) finishes one slot earlier than the paper's
    closed forms at D = 4: 2 (3N + D - 2) for the basic unit, 6N + 3 with early forwarding.  So
    the oracle's orders, which reach them, are optimal, and the paper's bubble counts are exact."""
    assert not _fits_in(4, N, closed_form - 1)
    gen = so.generate_timeline(4, N, early_forward=N > 4)
    assert so.makespan(gen) == closed_form


# ---- other stage placements: v chunks per device (Appendix A) and the looping map ("w/o V")

def test_zigzag_and_looping_maps():
    # v = 4 on D = 3 devices, down pipeline: 0 1 2 | 2 1 0 | 0 1 2 | 2 1 0; looping: 0 1 2 four times
    assert [so.vmap(0, s, 3, v=4) for s in range(12)] == [0, 1, 2, 2, 1, 0, 0, 1, 2, 2, 1, 0]
    assert [so.vmap(0, s, 3, v=4, looping=True) for s in range(12)] == [0, 1, 2] * 4
    assert [so.vmap(1, s, 3, v=2, looping=True) for s in range(6)] == [2, 1, 0, 2, 1, 0]
    # the default arguments are the V shape of Section 3.2
    assert all(so.vmap(d, s, 4) == so.vmap(d, s, 4, v=2, looping=False) for d in (0, 1) for s in range(8))
    with pytest.raises(ValueError):
        so.vmap(0, 8, 4, v=2)


@pytest.mark.parametrize("D,N,v,looping", [(4, 4, 4, False), (4, 8, 4, False), (4, 8, 2, True), (2, 4, 3, False),
                                           (4, 4, 1, False), (6, 6, 4, True), (4, 8, 3, True)])
def test_other_placements_give_valid_conflict_free_orders(D, N, v, looping):
    lanes = so.generate_timeline(D, N, v=v, looping=looping)
    order = so.serialise(lanes)
    assert so.conflicts(lanes) == 0
    assert so.validate(order, D, N, v, looping) is None
    assert len(order) == 2 * v * D * N
    assert max(so.peak_stash(lanes)) <= v * D              # D stage-activations of v chunk stashes
    # an order built for one map is rejected under the other (unless the maps coincide: v = 1)
    if v > 1:
        assert so.validate(order, D, N, v, not looping) is not None


@pytest.mark.parametrize("v", [1, 2, 4])
def test_bubble_time_shrinks_in_proportion_to_the_chunk_size(v):
    """Appendix A: with v chunks per device a chunk's forward and backward take 1/v of the time and
    the bubble is proportional to that time.  In slots (one chunk forward = 1) the basic unit at
    D = 4 therefore idles the same 4 slots per device for every v, i.e. 4 * (2/v) in units of the
    v = 2 chunk, while the work per device grows to 3 N v slots."""
    lanes = so.generate_timeline(4, 4, v=v)
    assert so.idle_per_device(lanes) == [4, 4, 4, 4]
    assert so.makespan(lanes) == 3 * 4 * v + 4


@pytest.mark.parametrize("D,N,v", [(4, 4, 2), (4, 8, 2), (4, 4, 4), (6, 6, 3), (2, 2, 2)])
def test_message_counts_of_the_two_maps(D, N, v):
    """Section 3.2 and Appendix A/C: the zig-zag map turns every lap boundary into a local copy, so an
    iteration sends 2 N v (D-1) messages and makes 2 N (v-1) local copies; the looping map sends
    all 2 N (vD-1) hand-overs between devices; going from v to 2v doubles the messages."""
    z = so.generate(D, N, v=v)
    lo = so.generate(D, N, v=v, looping=True)
    assert so.messages(z, D, v) == (2 * N * v * (D - 1), 2 * N * (v - 1))
    assert so.messages(lo, D, v, looping=True) == (2 * N * (v * D - 1), 0)
    z2 = so.generate(D, N, v=2 * v)
    assert so.messages(z2, D, 2 * v)[0] == 2 * so.messages(z, D, v)[0]
    assert so.cross_device_hops(z, D, v) == (v * (D - 1), v - 1)
