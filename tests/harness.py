"""Shared plumbing of the GPU parity tests: host<->device conversion, a thin wrapper that drives
the library through its C ABI, the matching oracle set-up, and the error metric."""
from __future__ import annotations

import numpy as np

import synth_inputs as si


def torch_mod():
    import torch
    return torch


def to_dev(arr, dtype):
    """float array -> device tensor holding the same values in the storage dtype."""
    torch = torch_mod()
    a = np.ascontiguousarray(arr, dtype=np.float32)
    if dtype == "bf16":
        bits = si.to_bf16_bits(a).view(np.int16)
        return torch.from_numpy(bits).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_host(t):
    """device tensor -> float64 numpy."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def empty_like_dev(shape, dtype):
    torch = torch_mod()
    return torch.empty(shape, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")


def rel_err(got, ref):
    """max|got-ref| / max|ref| (the parity metric), plus the l2 ratio for the report."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = max(np.max(np.abs(ref)), 1e-30)
    return float(np.max(np.abs(got - ref)) / den)


TOL = {"f32": 1e-4, "bf16": 2e-2}


class GpuStage:
    """Drives one library stage object for a StageConfig."""

    def __init__(self, cfg: si.StageConfig, max_inflight=0, wgrad_group=0, stash_recompute=0, forward_ahead=0):
        import paper_2410_19367_amd as bp
        self.bp = bp
        self.cfg = cfg
        self.h = bp.bp_stage_init_ex(cfg.layers, cfg.hidden, cfg.heads, cfg.seq, cfg.microbatch,
                                     cfg.causal, n_chunks=cfg.n_chunks, mlp=cfg.mlp,
                                     dtype=bp.BP_BF16 if cfg.dtype == "bf16" else bp.BP_F32,
                                     max_inflight=max_inflight, ln_eps=cfg.ln_eps,
                                     wgrad_group=wgrad_group, stash_recompute=stash_recompute,
                                     forward_ahead=forward_ahead)

    def close(self):
        if self.h is not None:
            self.bp.bp_stage_destroy(self.h)
            self.h = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def load_params(self, params):
        for c in range(self.cfg.n_chunks):
            for l in range(self.cfg.layers):
                for name, tid in self.bp.TENSOR_IDS.items():
                    self.bp.bp_stage_set_param(self.h, c, l, tid, params[c][l][name])

    def grad(self, chunk, layer, name):
        return self.bp.bp_stage_get_grad(self.h, chunk, layer, self.bp.TENSOR_IDS[name],
                                         si.param_shape(self.cfg, name)).astype(np.float64)

    def forward(self, chunk, mb, x_dev):
        out = empty_like_dev(tuple(x_dev.shape), self.cfg.dtype)
        self.bp.bp_stage_forward(self.h, chunk, mb, x_dev, out)
        return out

    def backward(self, chunk, mb, g_dev, direction=None):
        out = empty_like_dev(tuple(g_dev.shape), self.cfg.dtype)
        if direction is None:
            self.bp.bp_stage_backward(self.h, chunk, mb, g_dev, out)
        else:
            self.bp.bp_stage_backward_dir(self.h, chunk, mb, g_dev, out, direction)
        return out


def make_oracle(cfg: si.StageConfig, params):
    from oracle import stage_oracle as O
    st = O.StageOracle(cfg.layers, cfg.hidden, cfg.heads, cfg.seq, cfg.microbatch, cfg.causal,
                       n_chunks=cfg.n_chunks, mlp=cfg.mlp, ln_eps=cfg.ln_eps)
    st.load_params(params)
    return st


def run_fwd_bwd_parity(cfg: si.StageConfig, n_micro=None, seed=0, ln_jitter=0.0, check=True, wgrad_group=0,
                       stash_recompute=0, sync_each=True, grad_layers=None, forward_ahead=False):
    """F then B for each micro-batch on both sides; returns dict name -> rel err.
    sync_each=False: the GPU side runs all its micro-batches back to back with no device
    synchronisation in between (the call pattern bench.py times: consecutive calls overlap on the
    library's two streams); its outputs are kept on the device and compared afterwards.
    grad_layers: layers whose parameter gradients are compared (default: all).
    forward_ahead (with sync_each=False): the object runs its forwards on a stream of their own and
    the calls come in the order F(0) F(1) B(0) F(2) B(1) ..., so that the forward of one micro-batch
    overlaps the backward of the one before."""
    assert not (forward_ahead and sync_each)
    torch = torch_mod()
    n_micro = cfg.n_micro if n_micro is None else n_micro
    params = si.make_params(cfg, seed, ln_jitter)
    orc = make_oracle(cfg, params)
    errs = {}
    with GpuStage(cfg, wgrad_group=wgrad_group, stash_recompute=stash_recompute,
                  forward_ahead=int(forward_ahead)) as g:
        g.load_params(params)
        g.bp.bp_stage_zero_grad(g.h)
        kept = []
        if not sync_each:
            ins = []
            for mb in range(n_micro):
                lens = si.make_seqlens(cfg, mb, seed)
                if lens is not None:
                    g.bp.bp_stage_set_seqlens(g.h, mb, lens)
                ins.append((to_dev(si.make_activation(cfg, "act_in", mb, seed), cfg.dtype),
                            to_dev(si.make_activation(cfg, "grad_out", mb, seed), cfg.dtype)))
            torch.cuda.synchronize()
            if forward_ahead:
                zs = [g.forward(0, 0, ins[0][0])]
                for mb in range(n_micro):
                    if mb + 1 < n_micro:
                        zs.append(g.forward(0, mb + 1, ins[mb + 1][0]))
                    kept.append((zs[mb], g.backward(0, mb, ins[mb][1])))
                g.bp.bp_stage_wait_forward(g.h)
            else:
                for mb in range(n_micro):
                    z = g.forward(0, mb, ins[mb][0])
                    dx = g.backward(0, mb, ins[mb][1])
                    kept.append((z, dx))
            torch.cuda.synchronize()
        for mb in range(n_micro):
            x = si.make_activation(cfg, "act_in", mb, seed)
            go = si.make_activation(cfg, "grad_out", mb, seed)
            lens = si.make_seqlens(cfg, mb, seed)
            if lens is not None:
                if sync_each:
                    g.bp.bp_stage_set_seqlens(g.h, mb, lens)
                orc.set_seqlens(mb, lens)
            if sync_each:
                z = g.forward(0, mb, to_dev(x, cfg.dtype))
                dx = g.backward(0, mb, to_dev(go, cfg.dtype))
                torch.cuda.synchronize()
            else:
                z, dx = kept[mb]
            z_ref = orc.forward(0, mb, x)
            dx_ref = orc.backward(0, mb, go)
            errs[f"act_out[{mb}]"] = rel_err(to_host(z), z_ref)
            errs[f"grad_in[{mb}]"] = rel_err(to_host(dx), dx_ref)
            print(f"  parity {cfg.name}: micro-batch {mb} compared", flush=True)
        for l in (range(cfg.layers) if grad_layers is None else grad_layers):
            for name in si.PARAM_NAMES:
                errs[f"grad[{l}].{name}"] = rel_err(g.grad(0, l, name), orc.get_grad(0, l, name))
    if check:
        tol = TOL[cfg.dtype]
        bad = {k: v for k, v in errs.items() if not (v <= tol)}
        assert not bad, f"parity above {tol}: {bad}"
    return errs
