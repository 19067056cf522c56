"""GPU parity of the stage forward/backward against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest

import synth_inputs as si
from tests import harness as hz

pytestmark = pytest.mark.gpu


def test_cfg0_tiny_gpt_fp32_full():
    """Tiny GPT-style stage in fp32: all 4 micro-batches, gradients accumulated; bound 1e-4."""
    errs = hz.run_fwd_bwd_parity(si.CONFIGS[0])
    print({k: f"{v:.2e}" for k, v in errs.items()})


@pytest.mark.parametrize("name,kw", [
    ("gpt_d64", dict(layers=2, hidden=256, heads=4, seq=192, microbatch=2, causal=True)),
    ("gpt_d128_ragged", dict(layers=2, hidden=256, heads=2, seq=200, microbatch=1, causal=True)),
    ("bert_d64_padded", dict(layers=2, hidden=256, heads=4, seq=160, microbatch=3, causal=False,
                             len_lo=40, len_hi=160)),
    ("bert_full_len", dict(layers=1, hidden=128, heads=2, seq=96, microbatch=2, causal=False)),
    ("bert_d40_padded", dict(layers=2, hidden=320, heads=8, seq=128, microbatch=2, causal=False,
                             len_lo=40, len_hi=128)),
    ("gpt_d96", dict(layers=2, hidden=384, heads=4, seq=192, microbatch=1, causal=True)),
])
def test_small_bf16_stages(name, kw):
    cfg = si.scaled(si.CONFIGS[1], name="small_" + name, n_micro=2, **kw)
    errs = hz.run_fwd_bwd_parity(cfg, ln_jitter=0.1)
    worst = max(errs.items(), key=lambda kv: kv[1])
    print(name, "worst", worst)


@pytest.mark.parametrize("stash_recompute,wgrad_group,causal", [(0, 0, True), (1, 2, True), (0, 3, False)])
def test_forward_ahead_small_stages(stash_recompute, wgrad_group, causal):
    """Forwards on their own stream, one micro-batch ahead of the backwards (F0 F1 B0 F2 B1 ...), no
    synchronisation in between: outputs, input gradients and accumulated parameter gradients against
    the oracle, with the full and the reduced stash and with weight-gradient groups that end inside
    and at the end of the run."""
    kw = dict(layers=2, hidden=256, heads=4, seq=192, microbatch=2, causal=causal)
    if not causal:
        kw.update(len_lo=40, len_hi=192)
    cfg = si.scaled(si.CONFIGS[1], name="small_ahead", n_micro=5, **kw)
    hz.run_fwd_bwd_parity(cfg, ln_jitter=0.1, sync_each=False, forward_ahead=True,
                          stash_recompute=stash_recompute, wgrad_group=wgrad_group)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_forward_ahead_any_lead_gives_the_same_bits(seed):
    """Forwards up to three micro-batches ahead of the backwards, in a random but valid interleaving
    (backwards in micro-batch order, so the weight-gradient groups form the same way), three iterations
    on one object so that stash slots and group buffers are reused across the streams: every output and
    gradient equals, bit for bit, what the same object type gives in the plain order on one stream."""
    import torch
    rng = np.random.default_rng(seed)
    kw = [dict(layers=2, hidden=256, heads=4, seq=128, microbatch=2, causal=True),
          dict(layers=1, hidden=384, heads=4, seq=192, microbatch=1, causal=True),
          dict(layers=2, hidden=256, heads=2, seq=128, microbatch=3, causal=False, len_lo=30, len_hi=128)][seed]
    n_micro = 7
    cfg = si.scaled(si.CONFIGS[1], name="ahead_rand", n_micro=n_micro, **kw)
    params = si.make_params(cfg, seed, 0.1)
    ins = [(hz.to_dev(si.make_activation(cfg, "act_in", mb, seed), cfg.dtype),
            hz.to_dev(si.make_activation(cfg, "grad_out", mb, seed), cfg.dtype)) for mb in range(n_micro)]

    def calls(lead):
        order, f, b = [], 0, 0
        while b < n_micro:
            can_f = f < n_micro and f - b < lead
            if can_f and (f == b or rng.random() < 0.6):
                order.append(("F", f)); f += 1
            else:
                order.append(("B", b)); b += 1
        return order

    def run(forward_ahead, lead):
        with hz.GpuStage(cfg, max_inflight=4, wgrad_group=[3, 0, 2][seed], stash_recompute=int(seed == 1),
                         forward_ahead=forward_ahead) as g:
            g.load_params(params)
            for mb in range(n_micro):
                lens = si.make_seqlens(cfg, mb, seed)
                if lens is not None:
                    g.bp.bp_stage_set_seqlens(g.h, mb, lens)
            for it in range(3):
                g.bp.bp_stage_zero_grad(g.h)
                zs, dxs = {}, {}
                for kind, mb in calls(lead):
                    if kind == "F":
                        zs[mb] = g.forward(0, mb, ins[mb][0])
                    else:
                        dxs[mb] = g.backward(0, mb, ins[mb][1])
                g.bp.bp_stage_wait_forward(g.h)
            torch.cuda.synchronize()
            outs = [(hz.to_host(zs[mb]), hz.to_host(dxs[mb])) for mb in range(n_micro)]
            grads = {(l, n): g.grad(0, l, n) for l in range(cfg.layers) for n in si.PARAM_NAMES}
        return outs, grads

    outs_a, grads_a = run(1, 3)
    outs_b, grads_b = run(0, 1)
    for mb in range(n_micro):
        assert np.array_equal(outs_a[mb][0], outs_b[mb][0]), f"act_out[{mb}]"
        assert np.array_equal(outs_a[mb][1], outs_b[mb][1]), f"grad_in[{mb}]"
    for k in grads_a:
        assert np.array_equal(grads_a[k], grads_b[k]), k


def test_small_fp32_bert_padded():
    cfg = si.scaled(si.CONFIGS[0], name="small_f32_bert", causal=False, len_lo=10, len_hi=64,
                    microbatch=3, n_micro=2)
    hz.run_fwd_bwd_parity(cfg, ln_jitter=0.1)


def test_state_errors():
    import paper_2410_19367_amd as bp
    cfg = si.scaled(si.CONFIGS[0], name="state", layers=1)
    with hz.GpuStage(cfg, max_inflight=2) as g:
        x = hz.to_dev(si.make_activation(cfg, "act_in", 0), cfg.dtype)
        out = hz.empty_like_dev(tuple(x.shape), cfg.dtype)
        with pytest.raises(bp.BitPipeError) as e:
            bp.bp_stage_backward(g.h, 0, 0, x, out)
        assert e.value.code == bp.BP_ESTATE
        bp.bp_stage_forward(g.h, 0, 0, x, out)
        with pytest.raises(bp.BitPipeError) as e:
            bp.bp_stage_forward(g.h, 0, 0, x, out)
        assert e.value.code == bp.BP_ESTATE
        bp.bp_stage_forward(g.h, 0, 1, x, out)
        with pytest.raises(bp.BitPipeError) as e:      # max_inflight = 2
            bp.bp_stage_forward(g.h, 0, 2, x, out)
        assert e.value.code == bp.BP_ESTATE
        with pytest.raises(bp.BitPipeError) as e:
            bp.bp_stage_forward(g.h, 1, 0, x, out)
        assert e.value.code == bp.BP_EINVAL
        with pytest.raises(bp.BitPipeError) as e:
            bp.bp_stage_set_seqlens(g.h, 0, np.array([3, 3], dtype=np.int32))
        assert e.value.code == bp.BP_ESTATE       # causal stage
        bp.bp_stage_backward(g.h, 0, 1, x, out)
        bp.bp_stage_backward(g.h, 0, 0, x, out)
        with pytest.raises(bp.BitPipeError):
            bp.bp_stage_set_param(g.h, 0, 0, bp.TENSOR_IDS["wo"], np.zeros(7, dtype=np.float32))
    with pytest.raises(bp.BitPipeError) as e:
        bp.bp_stage_init(1, 100, 3, 8, 1, 1)
    assert e.value.code == bp.BP_ESHAPE


def test_zero_grad_semantics_across_iterations():
    """The clear between iterations: gradients read right after it are zero, an iteration after it
    reproduces the oracle's single-iteration gradients (nothing left over from the iteration
    before, nothing lost from the first micro-batch), and a second chunk that never ran a
    backward reads as zero."""
    cfg = si.scaled(si.CONFIGS[1], name="small_clear", layers=2, hidden=256, heads=2, seq=128,
                    microbatch=2, n_micro=3, n_chunks=2)
    params = si.make_params(cfg, 3, 0.1)
    orc = hz.make_oracle(cfg, params)
    with hz.GpuStage(cfg) as g:
        g.load_params(params)

        def iteration(seed, with_oracle):
            for mb in range(cfg.n_micro):
                x = si.make_activation(cfg, "act_in", mb, seed)
                go = si.make_activation(cfg, "grad_out", mb, seed)
                g.forward(0, mb, hz.to_dev(x, cfg.dtype))
                g.backward(0, mb, hz.to_dev(go, cfg.dtype))
                if with_oracle:
                    orc.forward(0, mb, x)
                    orc.backward(0, mb, go)

        iteration(11, False)                    # leaves non-zero gradients behind
        assert np.abs(g.grad(0, 1, "w1")).max() > 0
        g.bp.bp_stage_zero_grad(g.h)
        for name in si.PARAM_NAMES:
            assert not g.grad(0, 0, name).any(), name
        iteration(12, True)
        for l in range(cfg.layers):
            for name in si.PARAM_NAMES:
                err = hz.rel_err(g.grad(0, l, name), orc.get_grad(0, l, name))
                assert err <= hz.TOL[cfg.dtype], (l, name, err)
                assert not g.grad(1, l, name).any(), ("chunk 1 never ran", l, name)


@pytest.mark.parametrize("group,n_micro", [(1, 5), (2, 5), (3, 5), (4, 5), (5, 5), (8, 5), (8, 9)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_grouped_weight_gradients(group, n_micro, dtype):
    """Weight gradients computed over groups of 1..8 backward calls: the micro-batches give
    complete groups plus a remainder (or no complete group at all) that only the gradient
    read-out flushes; activations, input gradients and all accumulated gradients must match the
    oracle either way."""
    base = si.CONFIGS[1] if dtype == "bf16" else si.CONFIGS[0]
    cfg = si.scaled(base, name=f"small_group{group}_{n_micro}", layers=2, hidden=256, heads=2, seq=128,
                    microbatch=2, n_micro=n_micro, dtype=dtype, causal=True)
    hz.run_fwd_bwd_parity(cfg, ln_jitter=0.1, wgrad_group=group)


def test_grouped_weight_gradients_interleaved_chunks_and_directions():
    """Groups are kept per (chunk, direction): backward calls of two chunks and both directions
    interleave, with more stashes alive than any one group holds, and a clear in the middle of
    a group discards that group's waiting contributions."""
    cfg = si.scaled(si.CONFIGS[1], name="small_group_mix", layers=1, hidden=256, heads=2, seq=128,
                    microbatch=1, n_micro=5, n_chunks=2)
    params = si.make_params(cfg, 5, 0.1)
    orc = hz.make_oracle(cfg, params)
    with hz.GpuStage(cfg, max_inflight=12, wgrad_group=3) as g:
        g.load_params(params)
        xs = {mb: si.make_activation(cfg, "act_in", mb, 5) for mb in range(cfg.n_micro)}
        gos = {mb: si.make_activation(cfg, "grad_out", mb, 5) for mb in range(cfg.n_micro)}
        # a waiting contribution that the clear must discard
        g.forward(0, 0, hz.to_dev(xs[0], cfg.dtype))
        g.backward(0, 0, hz.to_dev(gos[0], cfg.dtype), direction=0)
        g.bp.bp_stage_zero_grad(g.h)
        for c in range(2):
            for mb in range(cfg.n_micro):
                g.forward(c, mb, hz.to_dev(xs[mb], cfg.dtype))
                orc.forward(c, mb, xs[mb])
        for mb in range(cfg.n_micro):
            for c in (1, 0):
                d = (mb + c) % 2
                g.backward(c, mb, hz.to_dev(gos[mb], cfg.dtype), direction=d)
                orc.backward(c, mb, gos[mb], d)
        # get_grad reads the direction-0 accumulators
        for c in range(2):
            for name in si.PARAM_NAMES:
                err = hz.rel_err(g.grad(c, 0, name), orc.grads[0][c][0][name])
                assert err <= hz.TOL[cfg.dtype], (c, name, err)
        # the sum of the two replicas (Section 3.4): direction 1 is added into direction 0, once
        for rep in range(2):
            g.bp.bp_stage_merge_directions(g.h)
            for c in range(2):
                for name in si.PARAM_NAMES:
                    want = orc.grads[0][c][0][name] + orc.grads[1][c][0][name]
                    err = hz.rel_err(g.grad(c, 0, name), want)
                    assert err <= hz.TOL[cfg.dtype], (rep, c, name, err)


@pytest.mark.parametrize("group", [1, 3, 5])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_lean_stash_recomputes_ln_and_gelu_outputs(group, dtype):
    """stash_recompute = 1 keeps 10 instead of 16 [T,H]-sized tensors per layer (Table 2's activation
    memory M_a) and rebuilds the LayerNorm and GELU outputs for the weight gradients: same
    activations, input gradients and accumulated gradients as the oracle, with and without
    grouped weight gradients (five micro-batches: complete groups and a flushed remainder)."""
    import paper_2410_19367_amd as bp
    base = si.CONFIGS[1] if dtype == "bf16" else si.CONFIGS[0]
    cfg = si.scaled(base, name=f"small_lean{group}", layers=2, hidden=256, heads=2, seq=128,
                    microbatch=2, n_micro=5, dtype=dtype, causal=True)
    hz.run_fwd_bwd_parity(cfg, ln_jitter=0.1, wgrad_group=group, stash_recompute=1)
    with hz.GpuStage(cfg) as full, hz.GpuStage(cfg, stash_recompute=1) as lean:
        esz = 2 if dtype == "bf16" else 4
        T, H, F = cfg.T, cfg.hidden, cfg.F
        saved = bp.bp_stage_stash_bytes(full.h) - bp.bp_stage_stash_bytes(lean.h)
        assert saved == cfg.layers * (2 * T * H + T * F) * esz          # a, m and g of every layer
        # 16 T H elements per layer plus the row statistics and the softmax log-sum-exp
        stats = (4 * T + cfg.microbatch * cfg.heads * cfg.seq) * 4
        assert bp.bp_stage_stash_bytes(full.h) == cfg.layers * (16 * T * H * esz + stats)
        assert bp.bp_stage_stash_bytes(lean.h) == cfg.layers * (10 * T * H * esz + stats)


def _random_small_configs(n, seed):
    """Seeded draw of small stage shapes that land on different kernel paths: aligned and ragged
    GEMMs, head widths 32..128 (some padded), causal / padded-bidirectional, MLP widths that are
    and are not multiples of 128, all weight-gradient group sizes, lean and full stash."""
    import random
    rng = random.Random(seed)
    out = []
    for i in range(n):
        d = rng.choice([32, 40, 64, 96, 128])
        heads = rng.choice([1, 2, 3, 4])
        hidden = d * heads
        causal = rng.random() < 0.5
        seq = rng.choice([64, 128, 192, 100, 72]) if d in (64, 128) or rng.random() < 0.7 else rng.choice([64, 128])
        mb = rng.choice([1, 2, 3])
        mlp = rng.choice([4 * hidden, 2 * hidden, 3 * hidden + 8, 512])
        kw = dict(layers=rng.choice([1, 2]), hidden=hidden, heads=heads, seq=seq, microbatch=mb, causal=causal,
                  mlp=mlp, n_micro=rng.choice([1, 2, 3, 5]))
        if not causal and rng.random() < 0.7:
            kw.update(len_lo=max(1, seq // 4), len_hi=seq)
        out.append((i, kw, rng.choice([1, 2, 3, 4]), rng.choice([0, 1])))
    return out


@pytest.mark.parametrize("idx,kw,group,lean", _random_small_configs(16, 20241127))
def test_random_small_stage_configs(idx, kw, group, lean):
    cfg = si.scaled(si.CONFIGS[1], name=f"small_rand{idx}", **kw)
    errs = hz.run_fwd_bwd_parity(cfg, ln_jitter=0.1, wgrad_group=group, stash_recompute=lean, seed=idx)
    worst = max(errs.items(), key=lambda kv: kv[1])
    print(idx, kw, "group", group, "lean", lean, "worst", worst)
