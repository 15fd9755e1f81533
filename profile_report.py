#!/usr/bin/env python3
"""Profiles a bench.py command with rocprofv3 and writes the summary kept under profiles/.

    python3 profile_report.py NAME [--sq] [--traffic KEY=KERNEL_SUBSTRING[@GRID]] -- <bench.py arguments>

runs, each as a process of its own under a time limit and stopping at the first failure,

    rocprofv3 --kernel-trace --stats          -- python3 bench.py <arguments>
    rocprofv3 --pmc FETCH_SIZE                -- python3 bench.py <arguments> --no-graph --copy-probe
    rocprofv3 --pmc WRITE_SIZE                -- python3 bench.py <arguments> --no-graph --copy-probe
    rocprofv3 --pmc <matrix-core counters>    -- python3 bench.py <arguments> --no-graph          (with --sq)

(raw output under gpurun_out/prof_NAME/) and turns the CSV files into profiles/NAME.md: the bench line of the
traced run, kernel times, HBM traffic per dispatch scaled by what the same counters read for a plain 1 GiB
device copy (--copy-probe), and with --sq the matrix-core busy fraction and the effective clock of every FFN kernel.
--traffic records the scaled bytes per launch of the named kernel (largest grid unless @GRID is given) in
profiles/traffic.json under KEY, together with a digest of the kernel sources, which bench.py copies into its
`roofline.traffic`.  `--report-only` skips the runs and rebuilds the summary from the CSV files already there.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
SQ_COUNTERS = ["SQ_VALU_MFMA_BUSY_CYCLES", "SQ_INSTS_VALU_MFMA_MOPS_BF16", "SQ_BUSY_CYCLES", "SQ_WAVE_CYCLES",
               "SQ_ACTIVE_INST_VALU", "SQ_ACTIVE_INST_LDS", "SQ_LDS_BANK_CONFLICT", "GRBM_GUI_ACTIVE"]
N_SIMD = 256 * 4        # MI355X: 256 compute units x 4 SIMDs
N_XCD = 8
COPY_KIB = 1 << 20      # the calibration copy moves 1 GiB


def short(name: str) -> str:
    name = name.replace("void ", "").replace("hmoe::", "")
    return name.split("(")[0][:90]


def run(cmd, log, limit):
    print("profile_report:", " ".join(cmd), flush=True)
    with open(log, "w") as fh:
        rc = subprocess.run(["timeout", "-s", "KILL", str(limit)] + cmd, stdout=fh, stderr=subprocess.STDOUT, cwd=ROOT,
                            env=dict(os.environ, TMPDIR="/tmp")).returncode
    if rc != 0:
        with open(log) as fh:
            print("".join(fh.readlines()[-15:]))
        raise SystemExit("profile_report: pass failed (exit %d), see %s" % (rc, log))


def counters(path):
    """-> {(kernel, grid): {counter: [value per dispatch]}}, {(kernel, grid): [duration ns]}"""
    vals = collections.defaultdict(lambda: collections.defaultdict(list))
    dur = collections.defaultdict(dict)
    with open(path) as fh:
        for r in csv.DictReader(fh):
            k = (short(r["Kernel_Name"]), int(r["Grid_Size"]))
            vals[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
            dur[k][r["Dispatch_Id"]] = int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
    return vals, {k: list(v.values()) for k, v in dur.items()}


def mean(v):
    return sum(v) / max(1, len(v))


def copies_report(args, out_dir, bench) -> int:
    """Transfer / compute overlap of the staging leg: kernel trace and memory-copy trace of one run."""
    full = ["rocprofv3", "--kernel-trace", "--memory-copy-trace", "--output-format", "csv", "-d", "gpurun_out/prof_" + args.name,
            "-o", "stg", "--"] + bench
    if not args.report_only:
        run(full, os.path.join(out_dir, "stg.log"), args.limit)
        for f in os.listdir(out_dir):
            if f.endswith(".db"):
                os.remove(os.path.join(out_dir, f))
    with open(os.path.join(out_dir, "stg_memory_copy_trace.csv")) as fh:
        copies = [(int(r["Start_Timestamp"]), int(r["End_Timestamp"])) for r in csv.DictReader(fh)
                  if "HOST_TO_DEVICE" in r["Direction"] and int(r["End_Timestamp"]) - int(r["Start_Timestamp"]) > 1000000]
    with open(os.path.join(out_dir, "stg_kernel_trace.csv")) as fh:
        kernels = [(int(r["Start_Timestamp"]), int(r["End_Timestamp"]), short(r["Kernel_Name"])) for r in csv.DictReader(fh)
                   if "ffn_" in r["Kernel_Name"]]
    copies.sort()
    total = under = hit = 0
    examples = []
    for k in kernels:
        total += k[1] - k[0]
        for c in copies:
            lo, hi = max(k[0], c[0]), min(k[1], c[1])
            if hi > lo:
                under += hi - lo
                hit += 1
                if len(examples) < 8:
                    examples.append((c, k))
                break
    md = ["# rocprofv3 summary: %s (staging copies against FFN kernels)" % args.name, "",
          "Written by `python3 profile_report.py %s --copies -- %s`, which runs" % (args.name, " ".join(args.bench_args)), "",
          "```", " ".join(full), "```", "",
          "Host-to-device copies longer than 1 ms (the staged experts): %d, %.2f ms on average, %.1f ms in total."
          % (len(copies), mean([c[1] - c[0] for c in copies]) / 1e6, sum(c[1] - c[0] for c in copies) / 1e6),
          "FFN kernel dispatches: %d, %.1f ms in total; %d of them ran while such a copy was in flight (%.2f ms of kernel time under "
          "a copy).  A copy waits for the last FFN call that read its slot and for nothing else, so it starts under the FFN of the "
          "experts that were resident (the slot it overwrites is not one they read) and the wave that needs it starts when it has "
          "landed; copies themselves run one after the other on the copy stream." % (len(kernels), total / 1e6, hit, under / 1e6), "",
          "Examples (ms from the start of the first listed copy):", "", "| copy | kernel | kernel runs |", "|---|---|---|"]
    t0 = examples[0][0][0] if examples else 0
    for c, k in examples:
        md.append("| %.3f .. %.3f | `%s` | %.3f .. %.3f |" % ((c[0] - t0) / 1e6, (c[1] - t0) / 1e6, k[2], (k[0] - t0) / 1e6, (k[1] - t0) / 1e6))
    if copies:
        first = copies[len(copies) // 2][0]
        ev = [(c[0], c[1], "copy host to device") for c in copies if first <= c[0] < first + 60_000_000]
        ev += [(k[0], k[1], "`%s`" % k[2]) for k in kernels if first - 1_000_000 <= k[0] < first + 60_000_000]
        md += ["", "A stretch of the timeline (ms):", "", "| start | end | what |", "|---|---|---|"]
        for e in sorted(ev)[:40]:
            md.append("| %.3f | %.3f | %s |" % ((e[0] - first) / 1e6, (e[1] - first) / 1e6, e[2]))
    with open(os.path.join(ROOT, "profiles", args.name + ".md"), "w") as fh:
        fh.write("\n".join(md) + "\n")
    print("profile_report: wrote profiles/%s.md" % args.name)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("name")
    ap.add_argument("--sq", action="store_true", help="also collect the matrix-core / sequencer counters")
    ap.add_argument("--traffic", action="append", default=[], help="KEY=KERNEL_SUBSTRING[@GRID]")
    ap.add_argument("--report-only", action="store_true")
    ap.add_argument("--copies", action="store_true",
                    help="a single pass with --kernel-trace --memory-copy-trace instead: which FFN kernels ran while a staging "
                         "copy (host to device, longer than 1 ms) was in flight")
    ap.add_argument("--limit", type=int, default=280, help="seconds per pass")
    argv = sys.argv[1:]
    cut = argv.index("--") if "--" in argv else len(argv)
    args = ap.parse_args(argv[:cut])
    args.bench_args = argv[cut + 1:]
    out_dir = os.path.join(ROOT, "gpurun_out", "prof_" + args.name)
    os.makedirs(out_dir, exist_ok=True)
    bench = ["python3", "bench.py"] + args.bench_args
    if args.copies:
        return copies_report(args, out_dir, bench)
    passes = [("trace", ["--kernel-trace", "--stats"], bench),
              ("fetch", ["--pmc", "FETCH_SIZE"], bench + ["--no-graph", "--copy-probe"]),
              ("write", ["--pmc", "WRITE_SIZE"], bench + ["--no-graph", "--copy-probe"])]
    if args.sq:
        passes.append(("sq", ["--pmc"] + SQ_COUNTERS, bench + ["--no-graph"]))
    commands = []
    digest_file = os.path.join(out_dir, "kernel_sources.txt")   # digest of the kernel sources that the passes ran with
    if not args.report_only:
        sys.path.insert(0, ROOT)
        from bench import kernel_sources_digest
        with open(digest_file, "w") as fh:
            fh.write(kernel_sources_digest() + "\n")
    for tag, opts, cmd in passes:
        full = ["rocprofv3"] + opts + ["--output-format", "csv", "-d", "gpurun_out/prof_" + args.name, "-o", tag, "--"] + cmd
        commands.append(" ".join(full))
        if not args.report_only:
            run(full, os.path.join(out_dir, tag + ".log"), args.limit)
            for f in os.listdir(out_dir):       # the raw databases are large and not needed for the summary
                if f.endswith(".db"):
                    os.remove(os.path.join(out_dir, f))

    md = ["# rocprofv3 summary: %s" % args.name, "",
          "Written by `python3 profile_report.py %s%s%s -- %s` (on the GPU box, from the repository root), which runs"
          % (args.name, " --sq" if args.sq else "", "".join(" --traffic " + t for t in args.traffic), " ".join(args.bench_args)),
          "", "```"] + commands + ["```", ""]
    with open(os.path.join(out_dir, "trace.log")) as fh:
        lines = [l for l in fh if l.startswith("{")]
    if lines:
        j = json.loads(lines[-1])
        roofline = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in j["roofline"].items()}
        md += ["Bench line of the traced run: `%s` %.0f %s, %.4f ms per step, roofline `%s`" %
               (j["config"]["workload"], j["value"], j["unit"], j["ms_per_step"], json.dumps(roofline)), ""]
        md += ["| phase | us per step (median, p10..p90) | gate/up us, fraction of binding roof | down us, fraction | layer fraction |",
               "|---|---|---|---|---|"]
        for ph, r in j["phases"].items():
            md.append("| %s | %.1f (%.1f..%.1f) | %.1f, %.3f %s | %.1f, %.3f %s | %.3f %s |" % (
                ph, r["ms_per_step"] * 1e3, r["ms_per_step_p10"] * 1e3, r["ms_per_step_p90"] * 1e3,
                r["gate_up"]["ms"] * 1e3, r["gate_up"]["frac"], r["gate_up"]["bound"],
                r["down"]["ms"] * 1e3, r["down"]["frac"], r["down"]["bound"], r["layer"]["frac"], r["layer"]["bound"]))
        md.append("")

    md += ["## Kernel time (`--kernel-trace --stats`)", "",
           "| kernel | calls | avg us | min us | max us | % of GPU time |", "|---|---|---|---|---|---|"]
    with open(os.path.join(out_dir, "trace_kernel_stats.csv")) as fh:
        for r in csv.DictReader(fh):
            if float(r["Percentage"]) >= 0.05:
                md.append("| `%s` | %s | %.1f | %.1f | %.1f | %.2f |" % (short(r["Name"]), r["Calls"], float(r["AverageNs"]) / 1e3,
                                                                       float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3,
                                                                       float(r["Percentage"])))
    # the trace pass replays HIP graphs, where kernels of the side stream overlap the others; per-grid averages of the
    # eager passes below time each launch shape separately
    fetch, fdur = counters(os.path.join(out_dir, "fetch_counter_collection.csv"))
    write, _ = counters(os.path.join(out_dir, "write_counter_collection.csv"))
    copies = [k for k in fetch if "copyBuffer" in k[0] and mean(write.get(k, {}).get("WRITE_SIZE", [0])) > 0.9 * COPY_KIB]
    f_scale = w_scale = 1.0
    if copies:
        f_scale = COPY_KIB / mean(fetch[copies[0]]["FETCH_SIZE"])
        w_scale = COPY_KIB / mean(write[copies[0]]["WRITE_SIZE"])
    md += ["", "## HBM traffic per dispatch (`--pmc FETCH_SIZE`, `--pmc WRITE_SIZE`, eager launches)", "",
           "Calibration: a plain 1 GiB device copy reads %.0f KiB on FETCH_SIZE and %.0f KiB on WRITE_SIZE, so the counters are "
           "scaled by %.3f and %.3f." % (COPY_KIB / f_scale, COPY_KIB / w_scale, f_scale, w_scale), "",
           "| kernel | grid (threads) | dispatches | avg us | FETCH_SIZE KiB | WRITE_SIZE KiB | scaled HBM bytes |",
           "|---|---|---|---|---|---|---|"]
    scaled = {}
    for k in fetch:
        fa, wa = mean(fetch[k]["FETCH_SIZE"]), mean(write.get(k, {}).get("WRITE_SIZE", [0]))
        scaled[k] = (f_scale * fa + w_scale * wa) * 1024
        if fa + wa >= 100 or "copy" in k[0].lower():
            md.append("| `%s` | %d | %d | %.1f | %.1f | %.1f | %.1f MB |" % (k[0], k[1], len(fetch[k]["FETCH_SIZE"]),
                                                                            mean(fdur[k]) / 1e3, fa, wa, scaled[k] / 1e6))
    if args.sq:
        sq, sdur = counters(os.path.join(out_dir, "sq_counter_collection.csv"))
        md += ["", "## Matrix-core counters of the FFN kernels (`--pmc %s`, eager launches)" % " ".join(SQ_COUNTERS), "",
               "MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / %d SIMDs / (GRBM_GUI_ACTIVE / %d dies); effective clock = (GRBM_GUI_ACTIVE / %d) "
               "/ duration; executed MFMA flops = 512 x SQ_INSTS_VALU_MFMA_MOPS_BF16." % (N_SIMD, N_XCD, N_XCD), "",
               "| kernel | grid | dispatches | avg us | cycles per die | effective GHz | MFMA busy | executed TFLOP per launch | "
               "executed TFLOP/s | VALU inst | LDS inst | LDS bank conflict cycles |", "|---|---|---|---|---|---|---|---|---|---|---|---|"]
        for k, c in sq.items():
            if "ffn_" not in k[0]:
                continue
            cyc = mean(c["GRBM_GUI_ACTIVE"]) / N_XCD
            us = mean(sdur[k]) / 1e3
            flop = 512.0 * mean(c["SQ_INSTS_VALU_MFMA_MOPS_BF16"])
            md.append("| `%s` | %d | %d | %.1f | %.0f | %.2f | %.3f | %.4f | %.0f | %.3g | %.3g | %.3g |" % (
                k[0], k[1], len(c["GRBM_GUI_ACTIVE"]), us, cyc, cyc / us / 1e3,
                mean(c["SQ_VALU_MFMA_BUSY_CYCLES"]) / N_SIMD / max(cyc, 1.0), flop / 1e12, flop / 1e12 / (us * 1e-6),
                mean(c["SQ_ACTIVE_INST_VALU"]), mean(c["SQ_ACTIVE_INST_LDS"]), mean(c["SQ_LDS_BANK_CONFLICT"])))
    with open(os.path.join(ROOT, "profiles", args.name + ".md"), "w") as fh:
        fh.write("\n".join(md) + "\n")
    print("profile_report: wrote profiles/%s.md" % args.name)

    if args.traffic:
        with open(digest_file) as fh:
            digest = fh.read().strip()
        path = os.path.join(ROOT, "profiles", "traffic.json")
        table = {}
        if os.path.exists(path):
            with open(path) as fh:
                table = json.load(fh)
        for spec in args.traffic:
            key, _, what = spec.partition("=")
            sub, _, grid = what.partition("@")
            cands = [k for k in scaled if sub in k[0] and (not grid or k[1] == int(grid))]
            if not cands:
                raise SystemExit("profile_report: no dispatch of a kernel matching %r" % what)
            k = max(cands, key=lambda c: c[1])
            table[key] = {"bytes": int(scaled[k]), "kernel": k[0], "grid": k[1], "sources": digest,
                          "profile": "profiles/%s.md" % args.name}
        with open(path, "w") as fh:
            json.dump(table, fh, indent=1, sort_keys=True)
            fh.write("\n")
        print("profile_report: updated profiles/traffic.json")
    return 0


if __name__ == "__main__":
    sys.exit(main())
