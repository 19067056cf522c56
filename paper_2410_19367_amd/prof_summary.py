#!/usr/bin/env python3
"""Turn rocprofv3 output (csv) into the short markdown summaries kept under profiles/.

    # per-kernel times of a run (rocprofv3 --kernel-trace --stats -d DIR -o NAME --output-format csv -- ...)
    python3 -m paper_2410_19367_amd.prof_summary stats DIR/NAME_kernel_stats.csv OUT.md \
        --title "..." --command "..." [--bench-log LOG]

    # hardware counters (one rocprofv3 --pmc run per pass, each with -o p --output-format csv):
    #   --pass-a : SQ_VALU_MFMA_BUSY_CYCLES GRBM_GUI_ACTIVE SQ_WAVE_CYCLES SQ_WAIT_ANY SQ_WAIT_INST_ANY
    #              SQ_WAIT_INST_LDS SQ_ACTIVE_INST_LDS SQ_BUSY_CYCLES
    #   --pass-b : SQ_INSTS_MFMA SQ_INSTS_LDS SQ_INSTS_VMEM_RD SQ_INSTS_VALU SQ_INSTS_SALU SQ_LDS_BANK_CONFLICT
    #              SQ_LDS_IDX_ACTIVE GRBM_GUI_ACTIVE
    #   --fetch / --write : FETCH_SIZE / WRITE_SIZE of the workload; --copy-fetch / --copy-write : the same
    #              two counters for `bench.py --copy-calibration` (a 1 GiB device-to-device copy)
    python3 -m paper_2410_19367_amd.prof_summary pmc OUT.md --workload NAME --title "..." --commands FILE \
        --pass-a DIR [--pass-b DIR] [--fetch DIR --write DIR --copy-fetch DIR --copy-write DIR]

Derived columns.  cycles = GRBM_GUI_ACTIVE / 8 (the counter is summed over the 8 XCDs);
clock = cycles / duration; MfmaUtil = SQ_VALU_MFMA_BUSY_CYCLES / (1024 SIMDs x cycles);
wait fractions are per wave cycle (SQ_WAIT_* / SQ_WAVE_CYCLES: ANY = waiting for anything, barrier
included; INST_ANY = an instruction's operands or issue; INST_LDS = LDS specifically).  FETCH_SIZE /
WRITE_SIZE are scaled by what the same counters read for the 1 GiB copy, so the byte figures are
traffic that leaves the L2s (to the Infinity Cache / HBM).
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re


def _short(name: str) -> str:
    name = name.replace("void bp::", "").replace("bp::", "")
    name = re.sub(r"\(bp::GemmArgs.*", "", name)
    name = re.sub(r"\(.*", "", name)
    return name[:96]


def cmd_stats(args):
    rows = list(csv.DictReader(open(args.csv)))
    out = [f"# {args.title}\n", "Command (from the repository root on the MI355X box):\n", f"    {args.command}\n",
           "| kernel | calls | total ms | avg us | min us | max us | % of GPU time |", "|---|---:|---:|---:|---:|---:|---:|"]
    gemm_ns = gemm_calls = 0
    for r in rows:
        name = r["Name"]
        if "gemm_" in name:
            gemm_ns += float(r["TotalDurationNs"])
            gemm_calls += int(r["Calls"])
        if "splitk_reduce" in name:
            gemm_ns += float(r["TotalDurationNs"])
        if float(r["Percentage"]) < 0.05:
            continue
        out.append(f"| `{_short(name)}` | {r['Calls']} | {float(r['TotalDurationNs']) / 1e6:.2f} | "
                   f"{float(r['AverageNs']) / 1e3:.1f} | {float(r['MinNs']) / 1e3:.1f} | {float(r['MaxNs']) / 1e3:.1f} | "
                   f"{float(r['Percentage']):.2f} |")
    out.append("")
    if gemm_calls:
        out.append(f"All GEMM launches together (a split-K GEMM counts as one launch, its reduce kernel's time "
                   f"included, as in bench.py's roofline object): {gemm_calls} launches, {gemm_ns / 1e6:.2f} ms, "
                   f"average {gemm_ns / gemm_calls / 1e3:.1f} us per launch.\n")
    if args.bench_log:
        lines = [l for l in open(args.bench_log) if l.startswith('{"metric"')]
        if lines:
            d = json.loads(lines[-1])
            keep = {k: d[k] for k in ("value", "unit", "ms_per_step", "ms_median", "ms_min", "tokens_per_s", "mfma_util",
                                      "t_bwd_over_t_fwd", "roofline") if k in d}
            out.append("bench.py line of this run (under the profiler), abridged:\n")
            out.append("    " + json.dumps(keep) + "\n")
            if "gemm_shapes" in d:
                out.append("GEMM launches of the event-timed pass by shape (bench.py `gemm_shapes`):\n")
                out.append("| M | N | K | form | epilogue | launches | avg us | TFLOP/s | share of GEMM time |")
                out.append("|---:|---:|---:|---|---|---:|---:|---:|---:|")
                for g in d["gemm_shapes"]:
                    out.append(f"| {g['M']} | {g['N']} | {g['K']} | {g['form'].split(' ')[0]} | {g['epilogue']} | "
                               f"{g['launches']} | {g['avg_us']} | {g['tflops']} | {g['share_of_gemm_time']} |")
                out.append("")
    open(args.out, "w").write("\n".join(out) + "\n")


def _load(d):
    """kernel -> counter -> [(value, duration ns)] per dispatch."""
    files = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit(f"no counter_collection.csv under {d}")
    out = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(files[0])):
        out[r["Kernel_Name"]][r["Counter_Name"]].append(
            (float(r["Counter_Value"]), int(r["End_Timestamp"]) - int(r["Start_Timestamp"])))
    return out


def _copy_scale(d, counter):
    """True KiB per counted unit, from the largest kernel of the 1 GiB copy run."""
    best = 0.0
    for k, v in _load(d).items():
        vals = v.get(counter, [])
        if vals:
            best = max(best, sum(x[0] for x in vals) / len(vals))
    return ((1 << 30) / 1024) / best if best else float("nan")


def cmd_pmc(args):
    A = _load(args.pass_a)
    Bc = _load(args.pass_b) if args.pass_b else {}
    have_bytes = bool(args.fetch and args.write and args.copy_fetch and args.copy_write)
    out = [f"# {args.title}\n", f"workload: {args.workload}\n",
           "Commands (from the repository root on the MI355X box, each pass a process of its own):\n"]
    out += ["    " + l.rstrip() for l in open(args.commands) if l.strip()]
    out.append("")
    out.append(__doc__.split("Derived columns.")[1].strip().replace("\n", " ") + "\n")
    f_scale = w_scale = None
    if have_bytes:
        Fd, Wd = _load(args.fetch), _load(args.write)
        f_scale, w_scale = _copy_scale(args.copy_fetch, "FETCH_SIZE"), _copy_scale(args.copy_write, "WRITE_SIZE")
        out.append(f"Copy calibration: one FETCH_SIZE unit = {f_scale:.4f} KiB, one WRITE_SIZE unit = {w_scale:.4f} KiB.\n")
    hdr = "| kernel | dispatches | avg us | clock GHz | MfmaUtil % | wait any | wait inst | wait LDS | LDS busy"
    sep = "|---|---:|---:|---:|---:|---:|---:|---:|---:"
    if Bc:
        hdr += " | LDS instr / MFMA | VMEM rd / MFMA | other VALU / MFMA | SALU / MFMA | bank conflicts"
        sep += "|---:|---:|---:|---:|---:"
    if have_bytes:
        hdr += " | fetch MB | write MB | TB/s beyond L2"
        sep += "|---:|---:|---:"
    rows = []
    tot_bytes, gemm_launches = 0.0, 0
    for k, c in A.items():
        g = c.get("GRBM_GUI_ACTIVE", [])
        if not g:
            continue
        n = len(g)
        cyc = sum(x[0] for x in g) / 8.0
        dur_us = sum(x[1] for x in g) / 1e3
        s = lambda name: sum(x[0] for x in c.get(name, []))
        wave = s("SQ_WAVE_CYCLES") or float("nan")
        line = (f"| `{_short(k)}` | {n} | {dur_us / n:.1f} | {cyc / dur_us / 1e3:.2f} | "
                f"{100 * s('SQ_VALU_MFMA_BUSY_CYCLES') / (1024 * cyc):.1f} | {s('SQ_WAIT_ANY') / wave:.2f} | "
                f"{s('SQ_WAIT_INST_ANY') / wave:.2f} | {s('SQ_WAIT_INST_LDS') / wave:.2f} | "
                f"{s('SQ_ACTIVE_INST_LDS') / (256 * cyc):.2f}")
        if Bc:
            b = Bc.get(k, {})
            sb = lambda name: sum(x[0] for x in b.get(name, []))
            mf = sb("SQ_INSTS_MFMA")
            if mf:
                act = sb("SQ_LDS_IDX_ACTIVE")
                line += (f" | {sb('SQ_INSTS_LDS') / mf:.2f} | {sb('SQ_INSTS_VMEM_RD') / mf:.2f} | "
                         f"{(sb('SQ_INSTS_VALU') - mf) / mf:.2f} | {sb('SQ_INSTS_SALU') / mf:.2f} | "
                         f"{(sb('SQ_LDS_BANK_CONFLICT') / act if act else 0):.3f}")
            else:
                line += " | - | - | - | - | -"
        if have_bytes:
            fv, wv = Fd.get(k, {}).get("FETCH_SIZE", []), Wd.get(k, {}).get("WRITE_SIZE", [])
            fe = sum(x[0] for x in fv) / max(len(fv), 1) * f_scale * 1024 / 1e6
            wr = sum(x[0] for x in wv) / max(len(wv), 1) * w_scale * 1024 / 1e6
            d2 = (sum(x[1] for x in fv) / len(fv) / 1e3) if fv else dur_us / n
            line += f" | {fe:.1f} | {wr:.1f} | {(fe + wr) / d2:.2f}"
            if "gemm_" in k or "splitk_reduce" in k:
                tot_bytes += (sum(x[0] for x in fv) * f_scale + sum(x[0] for x in wv) * w_scale) * 1024
                if "gemm_" in k:
                    gemm_launches += len(fv)
        rows.append((dur_us, line + " |"))
    out += [hdr + " |", sep + "|"]
    out += [r for _, r in sorted(rows, reverse=True)[:args.top]]
    out.append("")
    if have_bytes and gemm_launches:
        out.append(f"GEMM class (all gemm kernels plus the split-K reduction): {gemm_launches} launches, "
                   f"{tot_bytes / 1e6:.0f} MB beyond the L2s in total.\n")
        out.append(f"gemm_traffic_bytes_per_launch: {tot_bytes / gemm_launches:.0f}\n")
    if args.notes:
        out.append(open(args.notes).read())
    open(args.out, "w").write("\n".join(out) + "\n")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    s = sub.add_parser("stats")
    s.add_argument("csv"); s.add_argument("out")
    s.add_argument("--title", required=True); s.add_argument("--command", required=True); s.add_argument("--bench-log")
    p = sub.add_parser("pmc")
    p.add_argument("out")
    p.add_argument("--workload", required=True); p.add_argument("--title", required=True)
    p.add_argument("--commands", required=True, help="text file listing the commands that produced the passes")
    p.add_argument("--pass-a", required=True); p.add_argument("--pass-b")
    p.add_argument("--fetch"); p.add_argument("--write"); p.add_argument("--copy-fetch"); p.add_argument("--copy-write")
    p.add_argument("--notes", help="text file appended as the reading of the table")
    p.add_argument("--top", type=int, default=16)
    args = ap.parse_args()
    (cmd_stats if args.cmd == "stats" else cmd_pmc)(args)


if __name__ == "__main__":
    main()
