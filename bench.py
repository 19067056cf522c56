#!/usr/bin/env python3
"""Benchmark of the stage forward+backward hot path on one MI355X.

One step = one pass of the whole hot path over one batch of the workload: the chunk's forward and
backward for each of the config's micro-batches (weight gradients accumulated in fp32 across the
micro-batches), called as F(0) F(1) B(0) F(2) B(1) ... with the forwards on a stream of their own
(bp_opts.forward_ahead; `--plain-order`, and the widest workload by itself: F(0) B(0) F(1) B(1) ...
on one stream; `config.call_order` says which); for the V-schedule workload one whole BitPipe
iteration.  Inputs
are synthetic (seeded N(0,1) activations and upstream gradients, N(0,0.02) weights) and resident
in HBM before the timed region.

Prints ONE JSON line.  The headline (`value`, `roofline`, `cpu_baseline`) is the GPT-style stage
chunk the baseline file lists second (4 layers, H 2048, 8 micro-batches); the object `configs`
holds the same measurements for every other workload (BERT-style padded stage, the large GPT-style
stage, the whole V-schedule iteration, one stage of each of the paper's two models at their own
shapes), each with its own `roofline`.  Per workload:
  * `value`: TFLOP/s of algorithmic flops (72*T*H^2 + 12*T*S*H*c per layer and micro-batch) over
    the timed steps (mean); `ms_per_step`, `ms_median`, `ms_min` over the individually timed steps;
  * `tokens_per_s` (and, with key padding, `valid_tokens_per_s` and `value_valid_keys`, which count
    only unmasked tokens / keys, c_b = len_b / S);
  * `roofline`: the dominant kernel class, all bf16 MFMA GEMM launches, from HIP events recorded on
    the stage's stream around every launch in a second, equally long pass; `gemm_shapes` splits it
    by GEMM shape; `kernels` lists the other classes (attention against the MFMA peak, LayerNorm
    against the HBM peak);
  * `t_bwd_over_t_fwd`: backward time over forward time per micro-batch in that pass (the paper's
    cost model assumes 2, Section 3.3 / Appendix B);
  * `held_bytes_peak`: activation memory actually held at the peak (live stashes plus what open
    weight-gradient groups keep), next to `stash_bytes_per_microbatch` (the M_a of Table 2).
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2516.6     # MI355X dense bf16: 256 CUs x 4096 flop/clk x 2.4 GHz
HBM_PEAK_GBS = 8000.0
METRIC = "stage fwd+bwd TFLOP/s + MFMA util per micro-batch; tokens/s on 1 GPU"
# HBM-side bytes per GEMM launch (FETCH_SIZE + WRITE_SIZE of the GEMM kernels and their split-K
# reduce kernels, scaled by the plain-copy calibration), from the counter summaries under
# profiles/ that were collected with this same command: counters cannot be read from inside this
# process.  {workload: (bytes per launch, profile file)}; workloads without a summary report null.
GEMM_TRAFFIC = {}


def _load_traffic():
    """Read `gemm_traffic_bytes_per_launch` lines out of profiles/*_pmc_counters.md."""
    for path in glob.glob(os.path.join(ROOT, "profiles", "*_pmc_counters.md")):
        wl = val = None
        for line in open(path):
            if line.startswith("workload:"):
                wl = line.split(":", 1)[1].strip()
            if line.startswith("gemm_traffic_bytes_per_launch:"):
                val = float(line.split(":", 1)[1].split()[0])
        if wl and val:
            GEMM_TRAFFIC[wl] = (val, os.path.relpath(path, ROOT))


def _sclk_mhz():
    """Current shader clock from the driver's sysfs table (None if it cannot be read)."""
    for path in glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"):
        try:
            for line in open(path):
                if "*" in line:
                    return float(line.split(":")[1].strip().split("Mhz")[0].split("MHz")[0])
        except Exception:
            pass
    return None


def _time_steps(torch, step, steps, warmup):
    """warmup untimed steps, then `steps` steps timed one by one between device synchronisations.
    Returns (total seconds, per-step seconds)."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    per = []
    t_all = time.perf_counter()
    for _ in range(steps):
        t0 = time.perf_counter()
        step()
        torch.cuda.synchronize()
        per.append(time.perf_counter() - t0)
    return time.perf_counter() - t_all, per


def _roofline(cfg_name, gm, shapes):
    gemm_tflops = gm["flops"] / max(gm["ms"], 1e-9) / 1e9
    tr = GEMM_TRAFFIC.get(cfg_name)
    roof = {
        "kernel": "bf16 MFMA GEMM (forward, dgrad, wgrad of the four linear layers)",
        "bound": "mfma", "achieved": round(gemm_tflops, 3), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
        "frac": round(gemm_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "avg_launch_ms": round(gm["ms"] / max(gm["launches"], 1), 5), "launches": gm["launches"],
        "flops_per_launch": round(gm["flops"] / max(gm["launches"], 1), 1),
        "traffic": tr[0] if tr else None,
    }
    if tr:
        roof["traffic_source"] = tr[1]
    rows = []
    for sh in sorted(shapes, key=lambda s: -s["ms"]):
        fl = 2.0 * sh["M"] * sh["N"] * sh["K"] * sh["segments"] * sh["launches"]
        form = "wgrad" if sh["a_t"] else ("dgrad/fwd (both operands contraction-major)" if sh["b_t"] else "fwd")
        rows.append({"M": sh["M"], "N": sh["N"], "K": sh["K"] * sh["segments"], "form": form,
                     "epilogue": ["none", "bias+gelu", "gelu' + db partials"][sh["epilogue"]],
                     "launches": sh["launches"], "avg_us": round(sh["ms"] / max(sh["launches"], 1) * 1e3, 1),
                     "tflops": round(fl / max(sh["ms"], 1e-9) / 1e9, 1),
                     "share_of_gemm_time": round(sh["ms"] / max(gm["ms"], 1e-9), 3)})
    return roof, rows


def bench_stage(args, cfg, bp, si, torch, np, steps, warmup):
    def to_dev(a):
        a = np.ascontiguousarray(a, dtype=np.float32)
        if cfg.dtype == "bf16":
            return torch.from_numpy(si.to_bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    # Forwards one micro-batch ahead on their own stream fill the CUs that the start and the end of
    # every kernel leave idle: worth 5-12 % where kernels are short (cfg1, cfg2, cfg5, cfg6).  At
    # cfg3's size (single GEMMs of 0.5-3 ms) there is nothing to fill and two large GEMMs side by
    # side only disturb each other's L2 working sets (-2 %), so wide layers keep the plain order.
    plain = args.plain_order or 2.0 * cfg.T * cfg.hidden * cfg.F > 3e11
    st = bp.bp_stage_init_ex(cfg.layers, cfg.hidden, cfg.heads, cfg.seq, cfg.microbatch, cfg.causal,
                             n_chunks=1, mlp=cfg.mlp, dtype=bp.BP_BF16 if cfg.dtype == "bf16" else bp.BP_F32,
                             max_inflight=2, ln_eps=cfg.ln_eps, stash_recompute=int(args.stash_recompute),
                             wgrad_group=args.wgrad_group, forward_ahead=int(not plain))
    params = si.make_params(cfg, bulk=True)
    for l in range(cfg.layers):
        for name, tid in bp.TENSOR_IDS.items():
            bp.bp_stage_set_param(st, 0, l, tid, params[0][l][name])
    acts, gouts, all_lens = [], [], []
    for mb in range(cfg.n_micro):
        acts.append(to_dev(si.make_activation(cfg, "act_in", mb, bulk=True)))
        gouts.append(to_dev(si.make_activation(cfg, "grad_out", mb, bulk=True)))
        lens = si.make_seqlens(cfg, mb)
        if lens is not None:
            bp.bp_stage_set_seqlens(st, mb, lens)
            all_lens.append(lens)
    out = torch.empty_like(acts[0])
    gin = torch.empty_like(acts[0])

    outs = [out, torch.empty_like(out)]

    def step():
        bp.bp_stage_zero_grad(st)
        if plain:                   # F(0) B(0) F(1) B(1) ..., everything on the stage's stream
            for mb in range(cfg.n_micro):
                bp.bp_stage_forward(st, 0, mb, acts[mb], out)
                bp.bp_stage_backward(st, 0, mb, gouts[mb], gin)
            return
        # F(0) F(1) B(0) F(2) B(1) ...: the stage always has the next forward at hand, as in the
        # steady state of the schedule, and runs it beside the backward of the micro-batch before
        bp.bp_stage_forward(st, 0, 0, acts[0], outs[0])
        for mb in range(cfg.n_micro):
            if mb + 1 < cfg.n_micro:
                bp.bp_stage_forward(st, 0, mb + 1, acts[mb + 1], outs[(mb + 1) & 1])
            bp.bp_stage_backward(st, 0, mb, gouts[mb], gin)
        bp.bp_stage_wait_forward(st)

    bp.bp_stage_reset_peak_bytes(st)
    dt, per = _time_steps(torch, step, steps, warmup)
    sclk = _sclk_mhz()
    held = bp.bp_stage_held_bytes(st)
    flops_step = cfg.flops_per_microbatch() * cfg.n_micro
    tokens_step = cfg.T * cfg.n_micro
    tflops = flops_step * steps / dt / 1e12

    # second pass of the same steps with an event pair around every launch (one stream) and around
    # every forward / backward call
    bp.bp_prof_enable(st, 1)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks = []
    for _ in range(steps):
        bp.bp_stage_zero_grad(st)
        for mb in range(cfg.n_micro):
            a, b, c = ev(), ev(), ev()
            a.record()
            bp.bp_stage_forward(st, 0, mb, acts[mb], out)
            b.record()
            bp.bp_stage_backward(st, 0, mb, gouts[mb], gin)
            c.record()
            marks.append((a, b, c))
    prof = {name: bp.bp_prof_get(st, kid) for name, kid in bp.KERNEL_IDS.items()}
    shapes = bp.bp_prof_gemm_shapes(st)
    bp.bp_prof_enable(st, 0)
    torch.cuda.synchronize()
    t_f = sum(a.elapsed_time(b) for a, b, _ in marks) / len(marks)
    t_b = sum(b.elapsed_time(c) for _, b, c in marks) / len(marks)
    roof, gemm_rows = _roofline(cfg.name, prof["gemm"], shapes)
    kernels = {}
    for name, p in prof.items():
        if not p["launches"]:
            continue
        k = {"ms_per_step": p["ms"] / steps, "launches_per_step": p["launches"] // steps}
        if p["flops"]:
            k["tflops"] = p["flops"] / p["ms"] / 1e9
            k["frac_mfma_peak"] = k["tflops"] / MFMA_BF16_PEAK_TFLOPS
        if p["bytes"]:
            k["gbs"] = p["bytes"] / p["ms"] / 1e6
            k["frac_hbm_peak"] = k["gbs"] / HBM_PEAK_GBS
        kernels[name] = {a: (round(b, 4) if isinstance(b, float) else b) for a, b in k.items()}

    res = {
        "value": round(tflops, 3), "unit": "TFLOP/s", "steps": steps, "warmup": warmup,
        "ms_per_step": round(dt / steps * 1e3, 4),
        "ms_median": round(statistics.median(per) * 1e3, 4), "ms_min": round(min(per) * 1e3, 4),
        "value_at_ms_min": round(flops_step / min(per) / 1e12, 3),
        "dtype": cfg.dtype,
        "config": {"workload": cfg.name, "layers": cfg.layers, "hidden": cfg.hidden, "heads": cfg.heads,
                   "mlp": cfg.F, "seq": cfg.seq, "microbatch": cfg.microbatch, "causal": cfg.causal,
                   "micro_batches_per_step": cfg.n_micro,
                   "call_order": "F(0) B(0) F(1) B(1) ..., one stream" if plain else
                                 "F(0) F(1) B(0) F(2) B(1) ..., forwards on their own stream"},
        "tokens_per_s": round(tokens_step * steps / dt, 1),
        "ms_per_microbatch": round(dt / steps / cfg.n_micro * 1e3, 4),
        "mfma_util": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "t_fwd_ms": round(t_f, 4), "t_bwd_ms": round(t_b, 4), "t_bwd_over_t_fwd": round(t_b / max(t_f, 1e-9), 3),
        "stash_bytes_per_microbatch": bp.bp_stage_stash_bytes(st),
        "held_bytes_peak": held["peak_total"],
        "sclk_mhz_after_timed_steps": sclk,
        "roofline": roof, "gemm_shapes": gemm_rows, "kernels": kernels,
    }
    if all_lens:
        valid = float(sum(int(l.sum()) for l in all_lens))
        flops_valid = sum(cfg.flops_per_microbatch(l) for l in all_lens)
        res["valid_tokens_per_s"] = round(valid * steps / dt, 1)
        res["value_valid_keys"] = round(flops_valid * steps / dt / 1e12, 3)
        res["mean_valid_fraction"] = round(valid / tokens_step, 4)
    bp.bp_stage_destroy(st)
    return res, params


def bench_schedule(args, cfg, bp, si, torch, np, steps, warmup):
    """Whole BitPipe iteration (V-shaped bidirectional order, all virtual devices time-sliced on
    the one GPU): a step is one bp_run_schedule call over all micro-batches."""
    D = cfg.n_chunks // 2
    N = cfg.n_micro

    def to_dev(a):
        a = np.ascontiguousarray(a, dtype=np.float32)
        return torch.from_numpy(si.to_bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)

    st = bp.bp_stage_init_ex(cfg.layers, cfg.hidden, cfg.heads, cfg.seq, cfg.microbatch, cfg.causal,
                             n_chunks=cfg.n_chunks, mlp=cfg.mlp, dtype=bp.BP_BF16, ln_eps=cfg.ln_eps)
    params = si.make_params(cfg, bulk=True)
    for c in range(cfg.n_chunks):
        for l in range(cfg.layers):
            for name, tid in bp.TENSOR_IDS.items():
                bp.bp_stage_set_param(st, c, l, tid, params[c][l][name])
    inputs = to_dev(np.stack([si.make_activation(cfg, "act_in", m, bulk=True) for m in range(N)]))
    targets = to_dev(np.stack([si.make_activation(cfg, "target", m, bulk=True) for m in range(N)]))
    variant = 1 if args.order == "early" else 0
    order = bp.bp_schedule_generate(D, N, variant)
    model_ms, model_idle, model_peak = bp.bp_schedule_simulate(order, D, N)
    loss = [0.0]

    def step():
        loss[0] = bp.bp_run_schedule(st, order, D, inputs, targets)

    bp.bp_stage_reset_peak_bytes(st)
    dt, per = _time_steps(torch, step, steps, warmup)
    held = bp.bp_stage_held_bytes(st)
    flops_step = cfg.flops_per_microbatch() * cfg.n_chunks * N
    tflops = flops_step * steps / dt / 1e12
    bp.bp_prof_enable(st, 1)
    for _ in range(steps):
        step()
    gm = bp.bp_prof_get(st, bp.KERNEL_IDS["gemm"])
    shapes = bp.bp_prof_gemm_shapes(st)
    bp.bp_prof_enable(st, 0)
    roof, gemm_rows = _roofline(cfg.name, gm, shapes)
    res = {
        "value": round(tflops, 3), "unit": "TFLOP/s", "steps": steps, "warmup": warmup,
        "ms_per_step": round(dt / steps * 1e3, 4),
        "ms_median": round(statistics.median(per) * 1e3, 4), "ms_min": round(min(per) * 1e3, 4),
        "value_at_ms_min": round(flops_step / min(per) / 1e12, 3),
        "dtype": cfg.dtype,
        "config": {"workload": cfg.name, "stages": cfg.n_chunks, "virtual_devices": D, "layers_per_stage": cfg.layers,
                   "hidden": cfg.hidden, "heads": cfg.heads, "seq": cfg.seq, "microbatch": cfg.microbatch,
                   "micro_batches_per_step": N,
                   "order": "V-shaped bidirectional, " + ("early forwarding" if variant else "concatenated units")},
        # the same order replayed under the paper's cost model (chunk forward 1, backward 2, D devices)
        "cost_model": {"makespan": model_ms, "bubble_ratio": round(max(model_idle) / model_ms, 5),
                       "peak_chunk_stashes": max(model_peak)},
        "tokens_per_s": round(cfg.T * N * steps / dt, 1),
        "mfma_util": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "loss": round(float(loss[0]), 4),
        "stash_bytes_per_chunk_and_microbatch": bp.bp_stage_stash_bytes(st),
        "held_bytes_peak": held["peak_total"],
        "roofline": roof, "gemm_shapes": gemm_rows,
    }
    bp.bp_stage_destroy(st)
    return res, params


def cpu_baseline(cfg, params, si, np):
    """The oracle as it stands on a bounded sample (10-30 s of CPU work) of the workload: one
    micro-batch forward+backward, through the whole chunk for the 2048-wide configs, through one
    layer for the wider ones."""
    from oracle import stage_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    sample_layers = cfg.layers if cfg.hidden * cfg.T <= 2048 * 4096 else 1
    scfg = si.scaled(cfg, layers=sample_layers)
    orc = O.StageOracle(sample_layers, cfg.hidden, cfg.heads, cfg.seq, cfg.microbatch, cfg.causal,
                        mlp=cfg.mlp, ln_eps=cfg.ln_eps)
    orc.load_params([params[0][:sample_layers]])
    lens = si.make_seqlens(cfg, 0)
    if lens is not None:
        orc.set_seqlens(0, lens)
    x = si.make_activation(cfg, "act_in", 0, bulk=True)
    g = si.make_activation(cfg, "grad_out", 0, bulk=True)
    t0 = time.perf_counter()
    orc.forward(0, 0, x)
    orc.backward(0, 0, g)
    cdt = time.perf_counter() - t0
    return {
        "value": round(scfg.flops_per_microbatch() / cdt / 1e12, 5), "unit": "TFLOP/s", "cores": int(cores),
        "kind": "oracle",
        "sample": f"fp64 numpy oracle, 1 micro-batch fwd+bwd through {sample_layers} of the {cfg.layers} layers "
                  f"of {cfg.name} at full shape ({cdt:.1f} s)",
        "tokens_per_s": round(cfg.T * sample_layers / (cdt * cfg.layers), 2),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=None,
                    help="only this index into synth_inputs.CONFIGS (1..3: baseline stage configs; 4: whole "
                         "V-schedule iteration; 5, 6: stages of the paper's BERT-64 and GPT-96 at their own shapes); "
                         "default: headline on 1 plus all the others under `configs`")
    ap.add_argument("--order", choices=["concat", "early"], default="concat",
                    help="config 4 only: concatenated basic units or early forwarding")
    ap.add_argument("--stash-recompute", action="store_true",
                    help="stage configs: keep 10 instead of 16 [T,H] tensors per layer in the stash and "
                         "recompute the LayerNorm / GELU outputs for the weight gradients")
    ap.add_argument("--wgrad-group", type=int, default=0,
                    help="micro-batches per grouped weight-gradient GEMM (0: the library's default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--plain-order", action="store_true",
                    help="stage workloads: forward and backward of a micro-batch back to back on one stream "
                         "(default: forwards one micro-batch ahead on their own stream, bp_opts.forward_ahead)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy (reference for FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth_inputs as si
    import paper_2410_19367_amd as bp

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.copy_calibration:
        # a copy kernel of known size: reads 1 GiB and writes 1 GiB, five times
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_each_way": n, "repeats": 5}))
        return
    _load_traffic()

    def run(idx, steps, warmup):
        cfg = si.CONFIGS[idx]
        fn = bench_schedule if cfg.n_chunks > 1 else bench_stage
        return fn(args, cfg, bp, si, torch, np, steps, warmup)

    head_idx = 1 if args.config is None else args.config
    head, params = run(head_idx, args.steps, args.warmup)
    result = {"metric": METRIC, "value": head.pop("value"), "unit": head.pop("unit"), "n_gpus": 1,
              "steps": head.pop("steps"), "warmup": head.pop("warmup"), "ms_per_step": head.pop("ms_per_step"),
              "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head.pop("dtype"),
              "data": "synthetic"}
    result.update(head)
    if not args.no_cpu_baseline and si.CONFIGS[head_idx].n_chunks == 1:
        result["cpu_baseline"] = cpu_baseline(si.CONFIGS[head_idx], params, si, np)
    del params
    if args.config is None:
        others = {}
        for idx in (2, 3, 4, 5, 6):
            # the headline workload gets all the steps; the others half of them, the large stage (230 ms
            # per step) a quarter, which keeps the whole run within a couple of minutes
            steps = max(2, args.steps // 4) if idx == 3 else max(2, args.steps // 2)
            r, _ = run(idx, steps, min(args.warmup, 1) if idx == 3 else args.warmup)
            r.pop("kernels", None)
            others[si.CONFIGS[idx].name] = r
        result["configs"] = others
    print(json.dumps(result))


if __name__ == "__main__":
    main()
