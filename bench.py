#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all|mixtral|dsv2lite|qwen2moe|stress|toy]

A step is one pass of the whole hot path (router logits where the workload derives them from x,
route, permute, grouped expert FFN incl. shared experts, combine) over one batch of synthetic
tokens, inputs and the needed experts already resident in HBM.  With no --workload the run covers
every bf16 workload, one after the other (Mixtral-style decode 1 / 8 and prefill 512, DeepSeek-V2-Lite-
style decode 1 and prefill 1024, Qwen2-MoE-style decode 4 and prefill 2048, and the large-prefill stress
of 16384 tokens x 27 stacked layers), and prints ONE JSON line:

  * `value`: MoE-layer tokens/s of the largest workload (stress: 27 layers x 16384 tokens per step),
    the one the MFMA target is defined on; `roofline`: its dominant kernel (the routed experts' gate/up
    launch), timed inside this run with HIP events that the library records around that launch;
  * `phases`: every workload's phases with their gate/up, down and layer-level fractions of the HBM and
    the bf16 MFMA roof and the binding roof named; a phase is timed as `--blocks` blocks of K steps each
    and reports the median block (and p10 / p90);
  * `staging`: the same layers with the workload's real cache size, misses copied from pinned host memory
    (PCIe-inclusive figures, never part of `value`);
  * `cpu_baseline`: the CPU oracle timed on the host cores on a bounded sample of the headline batch.
"""
from __future__ import annotations

import argparse
import gc
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published

# phases per workload: (name, tokens); the last one is the workload's prefill batch
PHASES = {
    "toy": [("prefill16", 16)],
    "mixtral": [("decode1", 1), ("decode8", 8), ("prefill512", 512)],
    "dsv2lite": [("decode1", 1), ("prefill1024", 1024)],
    "qwen2moe": [("decode4", 4), ("prefill2048", 2048)],
    "stress": [("prefill16384", 16384)],
}
ALL = ["mixtral", "dsv2lite", "qwen2moe", "stress"]      # the default run, largest last: it is the headline
SEED0 = {"toy": 0, "mixtral": 1, "dsv2lite": 2, "qwen2moe": 3}
# sources of the kernels whose HBM traffic profiles/traffic.json records
TRAFFIC_SOURCES = ["ffn_tiled.hip", "tile_locate.h", "ffn_skinny.hip", "ffn_tiled_w4.hip", "common.h"]


def kernel_sources_digest() -> str:
    """Digest of the FFN kernel sources; profiles/traffic.json stores the one it was measured with."""
    h = hashlib.sha256()
    for name in TRAFFIC_SOURCES:
        with open(os.path.join(ROOT, "paper_2504_05897_amd", "csrc", name), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def roof(n_bytes: float, n_flops: float, ms: float) -> dict:
    """Fractions of the two roofs for `n_bytes` algorithmic bytes and `n_flops` algorithmic flops done in `ms`;
    the binding roof is the one whose minimum time is the larger."""
    if ms <= 0:
        return {"ms": 0.0}
    s = ms * 1e-3
    gbs, tfs = n_bytes / s / 1e9, n_flops / s / 1e12
    hbm, mfma = gbs / HBM_PEAK_GBS, tfs / MFMA_BF16_PEAK_TFLOPS
    return {"ms": ms, "GBps": gbs, "TFLOPs": tfs, "hbm_frac": hbm, "mfma_frac": mfma,
            "bound": "mfma" if mfma >= hbm else "hbm", "frac": max(hbm, mfma)}


def quantiles(v) -> dict:
    a = np.asarray(v, dtype=np.float64)
    return {"median": float(np.median(a)), "p10": float(np.percentile(a, 10)), "p90": float(np.percentile(a, 90)),
            "n": int(a.size)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="all", choices=["all"] + sorted(PHASES))
    ap.add_argument("--blocks", type=int, default=5, help="timed blocks of --steps steps per phase (median, p10, p90 over them)")
    ap.add_argument("--layers", type=int, default=0, help="stress: stacked layers (default 27); others: weight sets rotated (default 3)")
    ap.add_argument("--weights", default="bf16", choices=["bf16", "w4"],
                    help="w4: 4-bit group-wise expert weights (bf16 workloads)")
    ap.add_argument("--phase", default="", help="run only this phase of the workload (e.g. decode1), for profiling")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-staging", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a captured HIP graph")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB device copy three times (a kernel of known traffic, to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        return 2

    import torch
    import paper_2504_05897_amd as hm
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    w4 = args.weights == "w4"
    threads = min(16, len(os.sched_getaffinity(0)))
    blocks = max(1, args.blocks)
    names = ALL if args.workload == "all" else [args.workload]
    suffix = "+w4" if w4 else ""

    def to_dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(dev)
        return torch.from_numpy(a).to(dev)

    if args.copy_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def bench_workload(name: str):
        """-> (per-phase results, staging results or None, setup seconds, host copy of the first layer's inputs)"""
        shape = wl.SHAPES[name]
        bf16 = shape.dtype == wl.BF16
        assert bf16 or not w4, "4-bit weights go with bf16 activations"
        elem = 2 if bf16 else 4
        E, K, H, F = shape.n_experts, shape.top_k, shape.hidden, shape.ffn
        Fs = sum(shape.shared_ffn)
        stacked = name == "stress"
        # stress: the stacked layers are the step.  Others: weight sets taken in turn, so that a step cannot be
        # served from the 256 MB memory-side cache by the previous step's reads
        n_layers = args.layers or (27 if stacked else 3)
        phases = [p for p in PHASES[name] if not args.phase or p[0] == args.phase]
        assert phases, "workload %s has no phase %r" % (name, args.phase)
        w_bytes = (0.5 + 2.0 / 128) if w4 else elem   # bytes per stored expert weight (4-bit: codes + a bf16 scale per 128)
        max_T = max(t for _, t in phases)

        t0 = time.time()
        dtype_id = hm.HMOE_BF16_W4 if w4 else (hm.HMOE_BF16 if bf16 else hm.HMOE_F32)
        desc = hm.make_desc(H, F, E, K, E, dtype_id)          # all experts resident: the kernel-only figure
        layers, host_layers = [], []
        for li in range(n_layers):
            seed = (5000 + li) if stacked else SEED0[name] + 100 * li
            lay = wl.make_layer(shape, seed, max_T, threads=threads)
            layers.append(hm.MoELayer(desc, lay.experts, lay.shared, lay.w_router, max_tokens=max_T, host_copies=False))
            if li:
                lay.experts, lay.shared = [], []
            host_layers.append(lay)
        setup_s = time.time() - t0

        def run_phase(T):
            xs = [(to_dev(l.x[:T]), None if l.logits is None else to_dev(l.logits[:T])) for l in host_layers]
            stream = torch.cuda.current_stream()

            def one_step(i):
                if stacked:
                    for li in range(n_layers):
                        layers[li].forward(xs[li][0], xs[li][1])
                else:
                    li = i % n_layers
                    layers[li].forward(xs[li][0], xs[li][1])

            for i in range(max(args.warmup, n_layers)):
                one_step(i)
            torch.cuda.synchronize()
            timed_step = one_step
            if not args.no_graph:
                # the step is a fixed sequence of kernel launches: capture it once per weight set
                graphs = []
                for v in range(1 if stacked else n_layers):
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g):
                        one_step(v)
                    graphs.append(g)
                timed_step = lambda i: graphs[i % len(graphs)].replay()
                for i in range(args.warmup):
                    timed_step(i)
            torch.cuda.synchronize()
            block_ms = []
            for _ in range(blocks):              # each block: exactly --steps steps between two synchronised events
                ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                ev0.record(stream)
                for i in range(args.steps):
                    timed_step(i)
                ev1.record(stream)
                torch.cuda.synchronize()
                block_ms.append(ev0.elapsed_time(ev1) / args.steps)
            # second pass: HIP events around the two kernels of every FFN call, launched one after the other so
            # that each pair times one kernel alone (routed call first, then the shared experts' call)
            probe_steps = min(args.steps, 20)
            pairs_per_step = (n_layers if stacked else 1) * (4 if Fs else 2)
            saved = [(l.overlap_shared, l.merge_shared, l.merge_combine) for l in layers]
            for l in layers:
                l.overlap_shared = l.merge_shared = l.merge_combine = False
            hm.hmoe_probe_arm(probe_steps * pairs_per_step)
            for i in range(probe_steps):
                one_step(i)
            torch.cuda.synchronize()
            ms = hm.hmoe_probe_read(probe_steps * pairs_per_step)
            per_call = 4 if Fs else 2
            kern = {"gate_up": ms[0::per_call], "down": ms[1::per_call]}
            if Fs:
                kern["shared_gate_up"], kern["shared_down"] = ms[2::per_call], ms[3::per_call]
            if Fs and T <= 32 and not w4 and all(keep[1] for keep in saved):
                # third pass, decode-sized batches: the launches the timed steps really make there, which carry the
                # shared experts' FFN inside the routed experts' two launches
                for l in layers:
                    l.merge_shared = True
                merged_pairs = (n_layers if stacked else 1) * 2
                hm.hmoe_probe_arm(probe_steps * merged_pairs)
                for i in range(probe_steps):
                    one_step(i)
                torch.cuda.synchronize()
                ms = hm.hmoe_probe_read(probe_steps * merged_pairs)
                kern["gate_up_with_shared"], kern["down_with_shared"] = ms[0::2], ms[1::2]
            for l, keep in zip(layers, saved):
                l.overlap_shared, l.merge_shared, l.merge_combine = keep
            # what the routed kernels touched (distinct experts with rows, last step's routing)
            used = range(n_layers) if stacked else range(min(n_layers, probe_steps))
            distinct = float(np.mean([(np.diff(layers[li].offsets.cpu().numpy()) > 0).sum() for li in used]))
            return block_ms, {k: float(np.median(v)) for k, v in kern.items()}, distinct

        results = {}
        for pname, T in phases:
            block_ms, kern, distinct = run_phase(T)
            q = quantiles(block_ms)
            A = T * K
            per_step_layers = n_layers if stacked else 1
            per_layer_ms = q["median"] / per_step_layers
            # algorithmic work.  Routed gate/up: two of an expert's three matrices per distinct touched expert,
            # activations in, h out; 4 H F flops per assignment.  Down: the third matrix, h in, o_perm out.
            r = {
                "tokens": T, "layers_per_step": per_step_layers, "ms_per_step": q["median"], "ms_per_step_p10": q["p10"],
                "ms_per_step_p90": q["p90"], "blocks": q["n"], "tokens_per_s": T * per_step_layers / (q["median"] * 1e-3),
                "distinct_experts": distinct,
                "gate_up": roof(distinct * 2 * H * F * w_bytes + A * H * elem + A * F * elem, 4.0 * H * F * A, kern["gate_up"]),
                "down": roof(distinct * H * F * w_bytes + A * F * elem + A * H * elem, 2.0 * H * F * A, kern["down"]),
                "layer": roof(distinct * 3 * H * F * w_bytes + 3 * H * Fs * w_bytes, 6.0 * H * F * A + 6.0 * H * Fs * T, per_layer_ms),
            }
            if Fs:
                r["shared_gate_up"] = roof(2 * H * Fs * w_bytes + T * H * elem + T * Fs * elem, 4.0 * H * Fs * T, kern["shared_gate_up"])
                r["shared_down"] = roof(H * Fs * w_bytes + T * Fs * elem + T * H * elem, 2.0 * H * Fs * T, kern["shared_down"])
            if "gate_up_with_shared" in kern:   # the two launches of a decode step as it is timed: routed + shared work
                r["gate_up_with_shared"] = roof((distinct * F + Fs) * 2 * H * w_bytes + (A + T) * H * elem + (A * F + T * Fs) * elem,
                                                4.0 * H * (F * A + Fs * T), kern["gate_up_with_shared"])
                r["down_with_shared"] = roof((distinct * F + Fs) * H * w_bytes + (A * F + T * Fs) * elem + (A + T) * H * elem,
                                             2.0 * H * (F * A + Fs * T), kern["down_with_shared"])
            results[pname] = r

        # ---- staging: the workload's real cache size, misses copied from pinned host memory --------
        staging = None
        if not args.no_staging and shape.n_slots < E:
            lay0 = host_layers[0]
            d2 = hm.make_desc(H, F, E, K, shape.n_slots, dtype_id)
            for l in layers[1:]:
                l.close()
            del layers[1:]
            part = hm.MoELayer(d2, lay0.experts, lay0.shared, lay0.w_router, max_tokens=max_T)
            staging = {}
            for pname, T in phases:
                n_steps = 8
                xs = []
                for i in range(n_steps + 1):
                    lgi = wl.make_logits(shape, 777 + i, T)
                    xs.append((to_dev(wl.make_x(shape, 777 + i, T)), None if lgi is None else to_dev(lgi)))
                part.forward(*xs[0])
                torch.cuda.synchronize()
                part.staged_bytes = 0
                needed = hits = 0
                t1 = time.time()
                for i in range(1, n_steps + 1):
                    part.forward(*xs[i])
                    wave = part.last_plan[0]
                    needed += int((wave >= 0).sum())
                    hits += int((wave == 0).sum())
                torch.cuda.synchronize()
                dt = time.time() - t1
                staging[pname] = {"tokens_per_s_incl_pcie": T * n_steps / dt, "ms_per_step": dt / n_steps * 1e3,
                                  "hit_rate": hits / max(1, needed), "staged_GB_per_step": part.staged_bytes / n_steps / 1e9,
                                  "pcie_GBps_lower_bound": part.staged_bytes / dt / 1e9}
            # replacement policies on consecutive decode steps with temporal locality (Section IV-D, Fig. 8):
            # the same logit sequence served under LRU and under the score-aware policy of Eq. (3)
            pname, T = phases[0]
            if "decode" in pname:
                policies = {}
                n_seq, n_skip = 72, 8
                seq = wl.make_logit_sequence(shape, 4242, T, n_seq, 0.9)
                x_dev = to_dev(wl.make_x(shape, 4243, T))
                for pol_name, pol in (("lru", hm.HMOE_POLICY_LRU), ("mrs", hm.HMOE_POLICY_MRS)):
                    part.set_policy(pol, 0.5)
                    needed = hits = 0
                    for i in range(n_seq):
                        lg_dev = to_dev(seq[i])
                        part.forward(x_dev, lg_dev)
                        if pol == hm.HMOE_POLICY_MRS:
                            part.update_scores(lg_dev)
                        if i >= n_skip:     # the first steps only bring the cache from the other policy's state
                            wave = part.last_plan[0]
                            needed += int((wave >= 0).sum())
                            hits += int((wave == 0).sum())
                    policies[pol_name] = hits / max(1, needed)
                torch.cuda.synchronize()
                staging[pname]["hit_rate_correlated_steps"] = dict(policies, steps=n_seq - n_skip, rho=0.9, alpha=0.5)
            part.close()
            del part
        for l in layers:
            l.close()
        lay0 = host_layers[0]
        del layers, host_layers
        gc.collect()
        torch.cuda.empty_cache()
        if hasattr(torch._C, "_host_emptyCache"):
            torch._C._host_emptyCache()        # pinned host memory of the staging leg goes back as well
        return results, staging, setup_s, lay0, n_layers

    phases_out, staging_out, setup_out = {}, {}, {}
    head = None
    for name in names:
        results, staging, setup_s, lay0, n_layers = bench_workload(name)
        for pname, r in results.items():
            phases_out["%s/%s%s" % (name, pname, suffix)] = r
        if staging:
            for pname, r in staging.items():
                staging_out["%s/%s%s" % (name, pname, suffix)] = r
                # next to the kernel-only rate: the same phase with the workload's real cache size, copies included
                phases_out["%s/%s%s" % (name, pname, suffix)]["tokens_per_s_incl_pcie"] = r["tokens_per_s_incl_pcie"]
        setup_out[name] = setup_s
        head = (name, PHASES[name][-1] if not args.phase else [p for p in PHASES[name] if p[0] == args.phase][-1], lay0, n_layers)
        print("bench.py: %s done (setup %.1f s)" % (name, setup_s), file=sys.stderr, flush=True)

    head_name, (main_name, main_T), lay0, n_layers = head
    shape = wl.SHAPES[head_name]
    key = "%s/%s%s" % (head_name, main_name, suffix)
    main = phases_out[key]
    gu = main["gate_up"]
    if gu["bound"] == "mfma":
        roofline = {"bound": "mfma", "achieved": gu["TFLOPs"], "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": gu["mfma_frac"], "traffic": None}
    else:
        roofline = {"bound": "hbm", "achieved": gu["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gu["hbm_frac"],
                    "traffic": None}
    # HBM bytes per launch of that kernel from rocprofv3 FETCH_SIZE + WRITE_SIZE runs (profiles/, written by
    # profile_report.py together with a digest of the kernel sources they were measured with)
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(traffic_file):
        with open(traffic_file) as fh:
            table = json.load(fh)
        entry = table.get(key)
        if isinstance(entry, dict):
            roofline["traffic"] = entry.get("bytes")
            roofline["traffic_kernel"] = entry.get("kernel")
            roofline["traffic_sources_unchanged"] = entry.get("sources") == kernel_sources_digest()
    roofline["kernel"] = "ffn gate/up (routed experts), " + key
    roofline["kernel_ms"] = gu["ms"]

    # ---- CPU baseline: the oracle as it stands, bounded sample of the headline batch -------------
    cpu = None
    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_info, threadpool_limits
        from oracle import moe_oracle as orc
        sample = min(main_T, {"toy": 16, "mixtral": 512, "dsv2lite": 1024, "qwen2moe": 256, "stress": 512}[head_name])
        sub = np.arange(sample) * (main_T // sample)
        decode_weights = wl.as_f64
        if w4:      # the oracle's own quantiser: every weight replaced by the value its 4-bit code stands for
            from oracle import w4_oracle
            decode_weights = lambda m: w4_oracle.dequantize_w4(*w4_oracle.quantize_w4(wl.as_f32(m)))
        with threadpool_limits(limits=threads):     # the oracle's matrix products run in numpy's BLAS pool
            pools = [p for p in threadpool_info() if p.get("user_api") == "blas"]
            used = max([int(p["num_threads"]) for p in pools] or [1])
            if lay0.logits is None:
                logits = orc.router_logits(wl.as_f64(lay0.x[:main_T]), wl.as_f64(lay0.w_router))
            else:
                logits = lay0.logits[:main_T]
            t1 = time.time()
            reps = 0
            while True:                       # repeat until about 10 s of host work have been timed
                orc.moe_layer(wl.as_f64(lay0.x[:main_T]), logits, shape.top_k, lay0.experts, lay0.shared, token_subset=sub,
                              to_f64=decode_weights)
                reps += 1
                dt = time.time() - t1
                if dt >= 10.0 or reps >= 50:
                    break
        cpu = {"value": sample * reps / dt, "unit": "tokens/s", "cores": used, "kind": "oracle",
               "sample": "%d of the %d tokens of one %s layer (every %d-th), full layer in float64 numpy with %d BLAS threads, "
                         "%d repetitions in %.1f s" % (sample, main_T, key, main_T // sample, used, reps, dt)}

    out = {
        "metric": "MoE-layer tokens/s", "value": main["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": main["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": ("bf16 (4-bit weights)" if w4 else "bf16") if shape.dtype == wl.BF16 else "f32", "data": "synthetic",
        "config": {"workload": key, "hidden": shape.hidden, "ffn": shape.ffn, "experts": shape.n_experts, "top_k": shape.top_k,
                   "shared_ffn": list(shape.shared_ffn), "tokens": main_T, "layers": n_layers,
                   "launch": "eager" if args.no_graph else "hip-graph replay", "timed": "median of %d blocks of %d steps" % (blocks, args.steps),
                   "resident": "all needed experts resident in HBM slots (staging reported separately)"},
        "roofline": roofline, "cpu_baseline": cpu, "phases": phases_out, "staging": staging_out or None, "setup_s": setup_out,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
