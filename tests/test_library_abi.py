"""CPU-side checks of the shared library: it loads without a GPU, exports every symbol the
header declares, and its pure-CPU schedule functions agree with the schedule oracle."""
import os
import re

import pytest

import paper_2410_19367_amd as bp
from oracle import schedule_oracle as so

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "bitpipe_stage.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(bp_[a-z0-9_]+)\s*\(", header))
    assert declared == set(bp.binding.EXPORTS)
    lib = bp.binding.lib()
    for name in declared:
        assert hasattr(lib, name), name
    assert "gfx950" in bp.bp_version()


@pytest.mark.parametrize("D", [2, 4, 6, 8])
def test_vmap_agrees_with_oracle(D):
    for dr in (0, 1):
        for s in range(2 * D):
            assert bp.bp_schedule_vmap(dr, s, D) == so.vmap(dr, s, D)
    assert bp.bp_schedule_vmap(0, 2 * D, D) == -1
    assert bp.bp_schedule_vmap(2, 0, D) == -1


@pytest.mark.parametrize("D,N", [(2, 2), (2, 4), (4, 4), (4, 8), (4, 16), (6, 6), (6, 12), (8, 8), (8, 16), (10, 10), (12, 12),
                                 (16, 16)])
def test_generated_order_is_the_oracles(D, N):
    order = bp.bp_schedule_generate(D, N)
    assert bp.ops_to_tuples(order) == [tuple(o) for o in so.generate(D, N)]
    bp.bp_schedule_validate(order, D, N)
    lanes = so.generate_timeline(D, N)
    ms, idle, peak = bp.bp_schedule_simulate(order, D, N)
    assert ms <= so.makespan(lanes)
    assert max(peak) <= 2 * D


@pytest.mark.parametrize("D,N", [(2, 4), (4, 4), (4, 8), (4, 12), (4, 16), (6, 12), (8, 16)])
def test_early_forwarding_order_is_the_oracles(D, N):
    order = bp.bp_schedule_generate(D, N, variant=1)
    assert bp.ops_to_tuples(order) == [tuple(o) for o in so.generate(D, N, early_forward=True)]
    bp.bp_schedule_validate(order, D, N)


@pytest.mark.parametrize("D,N,v,looping,variant", [(4, 4, 4, 0, 0), (4, 8, 4, 0, 0), (4, 8, 2, 1, 0), (2, 4, 3, 0, 0),
                                                   (4, 4, 1, 0, 0), (6, 6, 4, 1, 0), (4, 8, 3, 1, 0), (4, 8, 4, 0, 1),
                                                   (4, 8, 2, 0, 1), (4, 4, 2, 0, 0)])
def test_other_layouts_agree_with_oracle(D, N, v, looping, variant):
    lay = bp.bp_layout(v, looping)
    for dr in (0, 1):
        for s in range(v * D):
            assert bp.bp_schedule_vmap_ex(lay, dr, s, D) == so.vmap(dr, s, D, v, bool(looping))
    assert bp.bp_schedule_vmap_ex(lay, 0, v * D, D) == -1
    order = bp.bp_schedule_generate_ex(lay, D, N, variant)
    ref = so.generate(D, N, early_forward=bool(variant), v=v, looping=bool(looping))
    assert bp.ops_to_tuples(order) == [tuple(o) for o in ref]
    bp.bp_schedule_validate_ex(lay, order, D, N)
    lanes = so.generate_timeline(D, N, early_forward=bool(variant), v=v, looping=bool(looping))
    ms, idle, peak = bp.bp_schedule_simulate_ex(lay, order, D, N)
    assert ms <= so.makespan(lanes)
    assert bp.bp_schedule_hops(lay, order, D, N) == so.messages(ref, D, v, bool(looping))
    if v > 1:       # the same ops do not fit the other map
        with pytest.raises(bp.BitPipeError) as e:
            bp.bp_schedule_validate_ex(bp.bp_layout(v, 1 - looping), order, D, N)
        assert e.value.code == bp.BP_EDEP


def test_layout_argument_checks():
    with pytest.raises(bp.BitPipeError) as e:
        bp.bp_schedule_generate_ex(bp.bp_layout(0, 0), 4, 4)
    assert e.value.code == bp.BP_EINVAL
    # the plain calls are the layout {2, 0}
    a = bp.ops_to_tuples(bp.bp_schedule_generate(4, 8))
    b = bp.ops_to_tuples(bp.bp_schedule_generate_ex(bp.bp_layout(2, 0), 4, 8))
    assert a == b


def test_simulate_reproduces_the_early_forwarding_closed_forms_at_D4():
    for N in (8, 12, 16):
        order = bp.bp_schedule_generate(4, N, variant=1)
        ms, idle, peak = bp.bp_schedule_simulate(order, 4, N)
        assert (ms, idle, max(peak)) == (6 * N + 3, [3, 3, 3, 3], 9)


def test_simulate_reproduces_the_closed_forms_at_D4():
    order = bp.bp_schedule_generate(4, 4)
    ms, idle, peak = bp.bp_schedule_simulate(order, 4, 4)
    assert (ms, idle, peak) == (28, [4, 4, 4, 4], [7, 8, 8, 7])


@pytest.mark.parametrize("D", [6, 8, 10, 12, 16])
def test_simulate_reproduces_the_basic_unit_closed_forms_beyond_D4(D):
    """Table 2 / Section 3.3 for N = D: makespan 2 (3N + D - 2) chunk slots, every device idle
    2 (D - 2) of them (ratio (D-2)/(3N+D-2)), at most D M_a = 2D chunk stashes."""
    order = bp.bp_schedule_generate(D, D)
    ms, idle, peak = bp.bp_schedule_simulate(order, D, D)
    assert ms == 8 * D - 4 and idle == [2 * (D - 2)] * D
    assert max(peak) == 2 * D and min(peak) >= D + 3


def test_generate_rejects_bad_arguments():
    for D, N in [(3, 3), (4, 6), (0, 4), (4, 2)]:
        with pytest.raises(bp.BitPipeError) as e:
            bp.bp_schedule_generate(D, N)
        assert e.value.code == bp.BP_EINVAL
    with pytest.raises(bp.BitPipeError):
        bp.bp_schedule_generate(4, 4, variant=7)


def test_validate_agrees_with_oracle_on_mutations():
    import random
    D, N = 4, 4
    good = bp.ops_to_tuples(bp.bp_schedule_generate(D, N))
    rng = random.Random(3)
    n_bad = 0
    for trial in range(200):
        t = list(good)
        kind = trial % 4
        if kind == 0:
            i, j = rng.randrange(len(t)), rng.randrange(len(t))
            t[i], t[j] = t[j], t[i]
        elif kind == 1:
            i = rng.randrange(len(t))
            t[i] = t[rng.randrange(len(t))]
        elif kind == 2:
            i = rng.randrange(len(t))
            k, d, v, s, m = t[i]
            t[i] = (k, d, (v + 1) % D, s, m)
        else:
            i = rng.randrange(len(t))
            k, d, v, s, m = t[i]
            t[i] = (k, 1 - d, D - 1 - v, s, m)
        want = so.validate([so.Op(*x) for x in t], D, N)
        try:
            bp.bp_schedule_validate(bp.ops_from_tuples(t), D, N)
            got_ok = True
        except bp.BitPipeError as e:
            assert e.code == bp.BP_EDEP
            got_ok = False
        assert got_ok == (want is None), (trial, want)
        n_bad += not got_ok
    assert n_bad > 100
    with pytest.raises(bp.BitPipeError):
        bp.bp_schedule_validate(bp.ops_from_tuples(good[:-1]), D, N)
