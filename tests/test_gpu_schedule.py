"""GPU parity of a whole BitPipe iteration (all virtual devices time-sliced on one GPU) against
the oracle's non-pipelined full-batch reference: loss and every accumulated gradient."""
import random

import numpy as np
import pytest

import synth_inputs as si
from oracle import schedule_oracle as so
from tests import harness as hz

pytestmark = pytest.mark.gpu


def _run_iteration(cfg, D, order_tuples=None, seed=0, expect_tol=None, layout=None, forward_ahead=0):
    import paper_2410_19367_amd as bp
    N = cfg.n_micro
    params = si.make_params(cfg, seed, ln_jitter=0.1)
    inputs = np.stack([si.make_activation(cfg, "act_in", m, seed) for m in range(N)])
    targets = np.stack([si.make_activation(cfg, "target", m, seed) for m in range(N)])
    lens = None
    if cfg.len_hi:
        lens = np.stack([si.make_seqlens(cfg, m, seed) for m in range(N)])
    orc = hz.make_oracle(cfg, params)
    loss_ref, G, _ = orc.full_batch_reference(inputs, targets, lens)
    with hz.GpuStage(cfg, forward_ahead=forward_ahead) as g:
        g.load_params(params)
        if lens is not None:
            for m in range(N):
                bp.bp_stage_set_seqlens(g.h, m, lens[m])
        if layout is None:
            order = bp.bp_schedule_generate(D, N) if order_tuples is None else bp.ops_from_tuples(order_tuples)
            loss = bp.bp_run_schedule(g.h, order, D, hz.to_dev(inputs, cfg.dtype), hz.to_dev(targets, cfg.dtype))
        else:
            lay = bp.bp_layout(*layout)
            order = bp.bp_schedule_generate_ex(lay, D, N)
            loss = bp.bp_run_schedule_ex(g.h, lay, order, D, hz.to_dev(inputs, cfg.dtype),
                                         hz.to_dev(targets, cfg.dtype))
        tol = expect_tol or hz.TOL[cfg.dtype]
        assert abs(loss - loss_ref) <= tol * abs(loss_ref), (loss, loss_ref)
        errs = {}
        for c in range(cfg.n_chunks):
            for l in range(cfg.layers):
                for name in si.PARAM_NAMES:
                    errs[(c, l, name)] = hz.rel_err(g.grad(c, l, name), G[c][l][name])
        bad = {k: v for k, v in errs.items() if not v <= tol}
        assert not bad, bad
        grads = {k: g.grad(*k) for k in errs}
    return loss, grads, max(errs.values())


def test_v_schedule_iteration_fp32_D2():
    cfg = si.scaled(si.CONFIGS[0], name="sched_f32", layers=1, n_chunks=4, n_micro=4, microbatch=1)
    _run_iteration(cfg, 2)


def test_iteration_on_an_object_with_forward_ahead_is_the_same():
    """bp_run_schedule orders its operations itself and leaves the object's forward stream alone: an
    object created with bp_opts.forward_ahead gives the same loss and the same gradient bits."""
    cfg = si.scaled(si.CONFIGS[4], name="sched_ahead", layers=1, hidden=128, heads=2, seq=128)
    loss_a, grads_a, _ = _run_iteration(cfg, 4, forward_ahead=1)
    loss_b, grads_b, _ = _run_iteration(cfg, 4, forward_ahead=0)
    assert loss_a == loss_b
    for k in grads_a:
        assert np.array_equal(grads_a[k], grads_b[k]), k


def test_v_schedule_iteration_bf16_D4_N8():
    """The topology of the V-schedule config (4 virtual devices x 2 chunks x 2 directions,
    8 micro-batches) at a reduced hidden size."""
    cfg = si.scaled(si.CONFIGS[4], name="sched_bf16", layers=1, hidden=128, heads=2, seq=128)
    loss, grads, worst = _run_iteration(cfg, 4)
    print("worst grad err", worst)


def test_early_forwarding_order_same_gradients_D4_N8():
    """Appendix B: the early-forwarding order only moves forwards ahead of time; executed on the GPU
    it must give the loss and gradients of the full-batch oracle, like the concatenated order."""
    import paper_2410_19367_amd as bp
    cfg = si.scaled(si.CONFIGS[4], name="sched_ef", layers=1, hidden=128, heads=2, seq=128)
    order = bp.ops_to_tuples(bp.bp_schedule_generate(4, cfg.n_micro, variant=1))
    assert order == [tuple(o) for o in so.generate(4, cfg.n_micro, early_forward=True)]
    loss_ef, grads_ef, worst = _run_iteration(cfg, 4, order_tuples=order)
    loss_cc, grads_cc, _ = _run_iteration(cfg, 4)
    assert abs(loss_ef - loss_cc) <= 1e-3 * abs(loss_cc)
    print("early forwarding worst grad err", worst)


@pytest.mark.parametrize("D,v,looping", [(2, 4, 0), (4, 2, 1), (2, 3, 1), (4, 1, 0)])
def test_other_layouts_same_gradients(D, v, looping):
    """Appendix A (more chunks per device) and the looping placement of the "w/o V" ablation run
    through the same executor: v*D stages, loss and gradients of the full-batch oracle."""
    cfg = si.scaled(si.CONFIGS[4], name=f"sched_v{v}_l{looping}", layers=1, hidden=128, heads=2, seq=64,
                    n_chunks=v * D, n_micro=2 * D)
    loss, grads, worst = _run_iteration(cfg, D, layout=(v, looping))
    print("layout", (D, v, looping), "worst grad err", worst)


def test_order_of_one_layout_is_rejected_under_another():
    import paper_2410_19367_amd as bp
    cfg = si.scaled(si.CONFIGS[0], name="sched_lay_bad", layers=1, n_chunks=8, n_micro=4, microbatch=1)
    with hz.GpuStage(cfg) as g:
        order = bp.bp_schedule_generate_ex(bp.bp_layout(2, 1), 4, 4)      # looping order
        x = hz.to_dev(np.zeros((4, cfg.microbatch, cfg.seq, cfg.hidden)), cfg.dtype)
        with pytest.raises(bp.BitPipeError) as e:
            bp.bp_run_schedule(g.h, order, 4, x, x)                        # executed as the V shape
        assert e.value.code == bp.BP_EDEP
        with pytest.raises(bp.BitPipeError) as e:                          # 8 chunks are not v*D = 16
            bp.bp_run_schedule_ex(g.h, bp.bp_layout(4, 0), bp.bp_schedule_generate_ex(bp.bp_layout(4, 0), 4, 4), 4, x, x)
        assert e.value.code == bp.BP_EINVAL


def test_v_schedule_iteration_bert_padded():
    cfg = si.scaled(si.CONFIGS[4], name="sched_bert", layers=1, hidden=128, heads=2, seq=96,
                    causal=False, len_lo=20, len_hi=96, n_chunks=4, n_micro=4, microbatch=2)
    _run_iteration(cfg, 2)


def test_any_valid_order_gives_the_same_gradients():
    cfg = si.scaled(si.CONFIGS[0], name="sched_order", layers=1, n_chunks=4, n_micro=4, microbatch=1)
    D, N = 2, 4
    base = so.generate(D, N)
    _, ref, _ = _run_iteration(cfg, D)
    rng = random.Random(5)
    pending, seen, order = list(base), set(), []
    while pending:
        ready = [o for o in pending if
                 (o.kind == "F" and (o.stage == 0 or ("F", o.stage - 1, o.mb) in seen)) or
                 (o.kind == "B" and ("F", o.stage, o.mb) in seen and
                  (o.stage == 2 * D - 1 or ("B", o.stage + 1, o.mb) in seen))]
        o = rng.choice(ready)
        pending.remove(o); seen.add((o.kind, o.stage, o.mb)); order.append(tuple(o))
    _, got, _ = _run_iteration(cfg, D, order_tuples=order)
    for k in ref:
        assert hz.rel_err(got[k], ref[k]) <= 1e-5, k      # fp32 accumulation order only


def test_invalid_order_is_rejected_before_any_launch():
    import paper_2410_19367_amd as bp
    cfg = si.scaled(si.CONFIGS[0], name="sched_bad", layers=1, n_chunks=4, n_micro=2, microbatch=1)
    D, N = 2, 2
    good = bp.ops_to_tuples(bp.bp_schedule_generate(D, N))
    i = next(k for k, o in enumerate(good) if o[0] == "B")
    bad = list(good)
    bad[0], bad[i] = bad[i], bad[0]
    with hz.GpuStage(cfg) as g:
        x = hz.to_dev(np.zeros((N, 1, cfg.seq, cfg.hidden)), cfg.dtype)
        with pytest.raises(bp.BitPipeError) as e:
            bp.bp_run_schedule(g.h, bp.ops_from_tuples(bad), D, x, x)
        assert e.value.code == bp.BP_EDEP
        with pytest.raises(bp.BitPipeError) as e:      # object holds 4 chunks, D = 4 needs 8
            bp.bp_run_schedule(g.h, bp.bp_schedule_generate(4, 4), 4, x, x)
        assert e.value.code == bp.BP_EINVAL
        # the object is still usable
        bp.bp_run_schedule(g.h, bp.ops_from_tuples(good), D, x, x)
