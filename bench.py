#!/usr/bin/env python3
"""Benchmark of the stage forward+backward hot path on one MI355X.

One step = one pass of the whole hot path over one batch of the workload: for each of the
config's micro-batches, the chunk's forward then its backward (weight gradients accumulated in
fp32 across the micro-batches).  Inputs are synthetic (seeded N(0,1) activations and upstream
gradients, N(0,0.02) weights) and resident in HBM before the timed region.

Prints ONE JSON line: whole-job throughput in TFLOP/s of algorithmic flops (72*T*H^2 +
12*T*S*H*c per layer per micro-batch), tokens/s, the roofline of the dominant kernel class (the
bf16 MFMA GEMMs) from HIP events recorded around each launch in a second, equally long pass,
and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16
HBM_PEAK_GBS = 8000.0
# Bytes that leave the L2s per GEMM launch (FETCH_SIZE + WRITE_SIZE of all GEMM kernels and their
# split-K reduce kernels, scaled by the plain-copy calibration, divided by the number of GEMM
# launches), from the hardware-counter passes over this same workload; counters cannot be read
# from inside this process, so the figure is carried over from
# profiles/stage_fwd_bwd_cfg1_pmc_counters.md.  Workloads without such a profile report null.
GEMM_TRAFFIC_BYTES_PER_LAUNCH = {"cfg1_gpt_h2048": 228.6e6}


def bench_schedule(args, cfg, bp, si, torch, np):
    """Whole BitPipe iteration (V-shaped bidirectional order, all virtual devices time-sliced on
    the one GPU): a step is one bp_run_schedule call over all micro-batches."""
    D = cfg.n_chunks // 2
    N = cfg.n_micro

    def to_dev(a):
        a = np.ascontiguousarray(a, dtype=np.float32)
        return torch.from_numpy(si.to_bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)

    st = bp.bp_stage_init_ex(cfg.layers, cfg.hidden, cfg.heads, cfg.seq, cfg.microbatch, cfg.causal,
                             n_chunks=cfg.n_chunks, mlp=cfg.mlp, dtype=bp.BP_BF16, ln_eps=cfg.ln_eps)
    params = si.make_params(cfg)
    for c in range(cfg.n_chunks):
        for l in range(cfg.layers):
            for name, tid in bp.TENSOR_IDS.items():
                bp.bp_stage_set_param(st, c, l, tid, params[c][l][name])
    inputs = to_dev(np.stack([si.make_activation(cfg, "act_in", m) for m in range(N)]))
    targets = to_dev(np.stack([si.make_activation(cfg, "target", m) for m in range(N)]))
    variant = 1 if args.order == "early" else 0
    order = bp.bp_schedule_generate(D, N, variant)
    model_ms, model_idle, model_peak = bp.bp_schedule_simulate(order, D, N)
    for _ in range(args.warmup):
        bp.bp_run_schedule(st, order, D, inputs, targets)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        loss = bp.bp_run_schedule(st, order, D, inputs, targets)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    flops_step = cfg.flops_per_microbatch() * cfg.n_chunks * N
    tflops = flops_step * args.steps / dt / 1e12
    bp.bp_prof_enable(st, 1)
    for _ in range(args.steps):
        bp.bp_run_schedule(st, order, D, inputs, targets)
    gm = bp.bp_prof_get(st, bp.KERNEL_IDS["gemm"])
    bp.bp_prof_enable(st, 0)
    gemm_tflops = gm["flops"] / max(gm["ms"], 1e-9) / 1e9
    result = {
        "metric": "stage fwd+bwd TFLOP/s + MFMA util per micro-batch; tokens/s on 1 GPU",
        "value": round(tflops, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(dt / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "stages": cfg.n_chunks, "virtual_devices": D, "layers_per_stage": cfg.layers,
                   "hidden": cfg.hidden, "heads": cfg.heads, "seq": cfg.seq, "microbatch": cfg.microbatch,
                   "micro_batches_per_step": N,
                   "order": "V-shaped bidirectional, " + ("early forwarding" if variant else "concatenated units")},
        # the same order replayed under the paper's cost model (chunk forward 1, backward 2, D devices)
        "cost_model": {"makespan": model_ms, "bubble_ratio": round(max(model_idle) / model_ms, 5),
                       "peak_chunk_stashes": max(model_peak)},
        "tokens_per_s": round(cfg.T * N * args.steps / dt, 1),
        "mfma_util": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "loss": round(float(loss), 4),
        "roofline": {"kernel": "bf16 MFMA GEMM (forward, dgrad, wgrad of the four linear layers)", "bound": "mfma",
                     "achieved": round(gemm_tflops, 3), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(gemm_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                     "avg_launch_ms": round(gm["ms"] / max(gm["launches"], 1), 5), "traffic": None},
    }
    bp.bp_stage_destroy(st)
    print(json.dumps(result))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=1, help="index into synth_inputs.CONFIGS (1..3: baseline stage configs; 4: whole V-schedule iteration; 5, 6: stages of the paper's BERT-64 and GPT-96 at their own shapes)")
    ap.add_argument("--order", choices=["concat", "early"], default="concat",
                    help="config 4 only: concatenated basic units or early forwarding")
    ap.add_argument("--stash-recompute", action="store_true",
                    help="stage configs: keep 10 instead of 16 [T,H] tensors per layer in the stash and "
                         "recompute the LayerNorm / GELU outputs for the weight gradients")
    ap.add_argument("--wgrad-group", type=int, default=0,
                    help="micro-batches per grouped weight-gradient GEMM (0: the library's default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
    cfg = si.CONFIGS[args.config]
    if cfg.n_chunks > 1:
        return bench_schedule(args, cfg, bp, si, torch, np)
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32

    def to_dev(a):
        a = np.ascontiguousarray(a, dtype=np.float32)
        if cfg.dtype == "bf16":
            return torch.from_numpy(si.to_bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    st = bp.bp_stage_init_ex(cfg.layers, cfg.hidden, cfg.heads, cfg.seq, cfg.microbatch, cfg.causal,
                             n_chunks=1, mlp=cfg.mlp, dtype=bp.BP_BF16 if cfg.dtype == "bf16" else bp.BP_F32,
                             max_inflight=2, ln_eps=cfg.ln_eps, stash_recompute=int(args.stash_recompute),
                             wgrad_group=args.wgrad_group)
    params = si.make_params(cfg)
    for l in range(cfg.layers):
        for name, tid in bp.TENSOR_IDS.items():
            bp.bp_stage_set_param(st, 0, l, tid, params[0][l][name])
    acts, gouts = [], []
    for mb in range(cfg.n_micro):
        acts.append(to_dev(si.make_activation(cfg, "act_in", mb)))
        gouts.append(to_dev(si.make_activation(cfg, "grad_out", mb)))
        lens = si.make_seqlens(cfg, mb)
        if lens is not None:
            bp.bp_stage_set_seqlens(st, mb, lens)
    out = torch.empty_like(acts[0])
    gin = torch.empty_like(acts[0])

    def step():
        bp.bp_stage_zero_grad(st)
        for mb in range(cfg.n_micro):
            bp.bp_stage_forward(st, 0, mb, acts[mb], out)
            bp.bp_stage_backward(st, 0, mb, gouts[mb], gin)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    flops_step = cfg.flops_per_microbatch() * cfg.n_micro
    tokens_step = cfg.T * cfg.n_micro
    ms_per_step = dt / args.steps * 1e3
    tflops = flops_step * args.steps / dt / 1e12

    # second pass of the same steps with an event pair around every launch
    bp.bp_prof_enable(st, 1)
    for _ in range(args.steps):
        step()
    prof = {name: bp.bp_prof_get(st, kid) for name, kid in bp.KERNEL_IDS.items()}
    bp.bp_prof_enable(st, 0)
    gm = prof["gemm"]
    gemm_avg_ms = gm["ms"] / max(gm["launches"], 1)
    gemm_tflops = gm["flops"] / max(gm["ms"], 1e-9) / 1e9
    kernels = {}
    for name, p in prof.items():
        if not p["launches"]:
            continue
        k = {"ms_per_step": p["ms"] / args.steps, "launches_per_step": p["launches"] // args.steps}
        if p["flops"]:
            k["tflops"] = p["flops"] / p["ms"] / 1e9
            k["frac_mfma_peak"] = k["tflops"] / MFMA_BF16_PEAK_TFLOPS
        if p["bytes"]:
            k["gbs"] = p["bytes"] / p["ms"] / 1e6
            k["frac_hbm_peak"] = k["gbs"] / HBM_PEAK_GBS
        kernels[name] = {a: (round(b, 4) if isinstance(b, float) else b) for a, b in k.items()}

    result = {
        "metric": "stage fwd+bwd TFLOP/s + MFMA util per micro-batch; tokens/s on 1 GPU",
        "value": round(tflops, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": cfg.name, "layers": cfg.layers, "hidden": cfg.hidden, "heads": cfg.heads,
                   "mlp": cfg.F, "seq": cfg.seq, "microbatch": cfg.microbatch, "causal": cfg.causal,
                   "micro_batches_per_step": cfg.n_micro},
        "tokens_per_s": round(tokens_step * args.steps / dt, 1),
        "ms_per_microbatch": round(ms_per_step / cfg.n_micro, 4),
        "stash_bytes_per_microbatch": bp.bp_stage_stash_bytes(st),
        "mfma_util": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "roofline": {
            "kernel": "bf16 MFMA GEMM (forward, dgrad, wgrad of the four linear layers)",
            "bound": "mfma",
            "achieved": round(gemm_tflops, 3),
            "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(gemm_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
            "avg_launch_ms": round(gemm_avg_ms, 5),
            "launches_per_step": gm["launches"] // args.steps,
            "traffic": GEMM_TRAFFIC_BYTES_PER_LAUNCH.get(cfg.name),
        },
        "kernels": kernels,
    }

    if not args.no_cpu_baseline:
        from oracle import stage_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        # bounded sample (10-30 s of CPU work): one micro-batch through the whole chunk for the
        # 2048-wide configs, through one layer for the wider ones
        sample_layers = cfg.layers if cfg.hidden * cfg.T <= 2048 * 4096 else 1
        scfg = si.scaled(cfg, layers=sample_layers)
        orc = O.StageOracle(sample_layers, cfg.hidden, cfg.heads, cfg.seq, cfg.microbatch, cfg.causal,
                            mlp=cfg.mlp, ln_eps=cfg.ln_eps)
        orc.load_params([params[0][:sample_layers]])
        lens = si.make_seqlens(cfg, 0)
        if lens is not None:
            orc.set_seqlens(0, lens)
        x = si.make_activation(cfg, "act_in", 0)
        g = si.make_activation(cfg, "grad_out", 0)
        t0 = time.perf_counter()
        orc.forward(0, 0, x)
        orc.backward(0, 0, g)
        cdt = time.perf_counter() - t0
        result["cpu_baseline"] = {
            "value": round(scfg.flops_per_microbatch() / cdt / 1e12, 5),
            "unit": "TFLOP/s",
            "cores": int(cores),
            "kind": "oracle",
            "sample": f"fp64 numpy oracle, 1 micro-batch fwd+bwd through {sample_layers} of the {cfg.layers} layers "
                      f"at full shape ({cdt:.1f} s)",
            "tokens_per_s": round(cfg.T * sample_layers / (cdt * cfg.layers), 2),
        }

    bp.bp_stage_destroy(st)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
