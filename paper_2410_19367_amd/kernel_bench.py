#!/usr/bin/env python3
"""Time single kernels of the stage library at a workload's shapes (and give rocprofv3 something
small to profile): the linear-layer GEMMs in their three forms, through the C ABI's bp_op_* calls.

    python3 -m paper_2410_19367_amd.kernel_bench --config 3              # every GEMM of the config
    python3 -m paper_2410_19367_amd.kernel_bench --gemm nt 4096 20480 5120 --loops 1
    python3 -m paper_2410_19367_amd.kernel_bench --config 1 --vendor     # same shapes through torch.matmul

Forms: `nt` = both operands contraction-major (the library's forward and data-gradient GEMMs, which
read a transposed weight copy), `tn` = weight gradient dW += X^T dY over `--segments` micro-batches.
Timing: half the iterations untimed, then a loop of about 40 ms between two events on the stream
(long enough for the shader clock to settle under load).  `--vendor` times torch.matmul on the same
operands: the vendor library's rate on this machine, as context for the roofline fractions.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _time(torch, f, flops, loops=None):
    iters = loops or max(10, int(40e-3 / (flops / 1.0e15)))
    for _ in range(max(1, iters // 2)):
        f()
    torch.cuda.synchronize()
    s = torch.cuda.Event(enable_timing=True)
    e = torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(iters):
        f()
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) / iters


def gemm_case(bp, torch, form, M, N, K, segments=1, vendor=False, loops=None):
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    rnd = lambda *shape: torch.randn(*shape, device="cuda", generator=g).bfloat16()
    if form == "nt":        # C[M,N] = A[M,K] B[N,K]^T
        A, B = rnd(M, K), rnd(N, K)
        C = torch.empty(M, N, device="cuda", dtype=torch.bfloat16)
        if vendor:
            f = lambda: torch.matmul(A, B.t(), out=C)
        else:
            f = lambda: bp.bp_op_gemm(bp.BP_BF16, 0, 1, M, N, K, A, K, B, K, C, N)
        flops = 2.0 * M * N * K
    elif form == "tn":      # dW[M,N] += sum_i X_i[K,M]^T dY_i[K,N]
        Xs = [rnd(K, M) for _ in range(segments)]
        Ys = [rnd(K, N) for _ in range(segments)]
        W = torch.zeros(M, N, device="cuda")
        ws = torch.empty(min(4 * M * N, 64 << 20), device="cuda")
        if vendor:
            Xc, Yc = torch.cat(Xs), torch.cat(Ys)
            f = lambda: torch.matmul(Xc.t(), Yc)
        else:
            f = lambda: bp.bp_op_wgrad_group(bp.BP_BF16, M, N, K, Xs, Ys, W, 0, ws, ws.numel())
        flops = 2.0 * M * N * K * segments
    else:
        raise ValueError(form)
    ms = _time(torch, f, flops, loops)
    who = "vendor " if vendor else ""
    print(f"{who}{form} M={M:6d} N={N:6d} K={K * segments:6d}  {ms * 1e3:9.1f} us  {flops / ms / 1e9:8.1f} TFLOP/s", flush=True)
    return ms


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, default=None, help="index into synth_inputs.CONFIGS: time every GEMM of one layer")
    ap.add_argument("--gemm", nargs=4, metavar=("FORM", "M", "N", "K"), help="one GEMM: nt | tn and its sizes")
    ap.add_argument("--segments", type=int, default=1, help="tn: micro-batches per grouped weight gradient")
    ap.add_argument("--vendor", action="store_true", help="time torch.matmul instead of this library")
    ap.add_argument("--loops", type=int, default=None, help="timed iterations (default: about 40 ms worth)")
    args = ap.parse_args()
    import torch
    import synth_inputs as si
    import paper_2410_19367_amd as bp
    if not torch.cuda.is_available():
        print("kernel_bench: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.gemm:
        form, M, N, K = args.gemm[0], int(args.gemm[1]), int(args.gemm[2]), int(args.gemm[3])
        gemm_case(bp, torch, form, M, N, K, args.segments, args.vendor, args.loops)
        return
    cfg = si.CONFIGS[1 if args.config is None else args.config]
    T, H, F = cfg.T, cfg.hidden, cfg.F
    group = min(8, max(1, 16384 // T))
    print(f"# {cfg.name}: T={T} H={H} F={F}, weight gradients over {group} micro-batches", flush=True)
    for n, k in ((3 * H, H), (H, H), (F, H), (H, F)):
        gemm_case(bp, torch, "nt", T, n, k, 1, args.vendor, args.loops)      # forward
        gemm_case(bp, torch, "nt", T, k, n, 1, args.vendor, args.loops)      # data gradient
        gemm_case(bp, torch, "tn", k, n, T, group, args.vendor, args.loops)  # weight gradient


if __name__ == "__main__":
    main()
