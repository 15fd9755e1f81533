#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload mixtral|dsv2lite|qwen2moe|stress|toy]

A step is one pass of the whole hot path (router logits where the workload derives them from x,
route, permute, grouped expert FFN incl. shared experts, combine) over one batch of synthetic
tokens, inputs and the needed experts already resident in HBM.  Prints ONE JSON line:
MoE-layer tokens/s for the workload's prefill batch (`value`), the per-phase results, the roofline
of the dominant kernel (gate/up FFN) measured with HIP events around that kernel inside this run,
and the CPU oracle timed on the host cores as a reported baseline.
"""
from __future__ import annotations

import argparse
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

# phases per workload: (name, tokens); the last one is the prefill batch reported as `value`
PHASES = {
    "toy": [("prefill16", 16)],
    "mixtral": [("decode1", 1), ("decode8", 8), ("prefill512", 512)],
    "dsv2lite": [("decode1", 1), ("prefill1024", 1024)],
    "qwen2moe": [("decode4", 4), ("prefill2048", 2048)],
    "stress": [("prefill16384", 16384)],
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="mixtral", choices=sorted(PHASES))
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
    shape = wl.SHAPES[args.workload]
    bf16 = shape.dtype == wl.BF16
    elem = 2 if bf16 else 4
    E, K, H, F = shape.n_experts, shape.top_k, shape.hidden, shape.ffn
    Fs = sum(shape.shared_ffn)
    # stress: the 27 stacked layers are the step.  Others: three weight sets taken in turn, so that a step
    # cannot be served from the 256 MB memory-side cache by the previous step's reads
    n_layers = args.layers or (27 if args.workload == "stress" else 3)
    phases = [p for p in PHASES[args.workload] if not args.phase or p[0] == args.phase]
    w4 = args.weights == "w4"
    if w4:
        assert bf16, "4-bit weights go with bf16 activations"
    w_bytes = (0.5 + 2.0 / 128) if w4 else elem      # bytes per stored expert weight (4-bit: codes + one bf16 scale per 128)
    assert phases, "workload %s has no phase %r" % (args.workload, args.phase)
    max_T = max(t for _, t in phases)
    threads = min(16, len(os.sched_getaffinity(0)))

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

    # ---- layers: all experts resident for the kernel-only figure ------------------------------
    t0 = time.time()
    dtype_id = hm.HMOE_BF16_W4 if w4 else (hm.HMOE_BF16 if bf16 else hm.HMOE_F32)
    desc = hm.make_desc(H, F, E, K, E, dtype_id)
    layers, host_layers = [], []
    for li in range(n_layers):
        seed = (5000 + li) if args.workload == "stress" else {"toy": 0, "mixtral": 1, "dsv2lite": 2, "qwen2moe": 3}[args.workload] + 100 * li
        lay = wl.make_layer(shape, seed, max_T, threads=threads)
        layers.append(hm.MoELayer(desc, lay.experts, lay.shared, lay.w_router, max_tokens=max_T))
        if li == 0:
            host_layers.append(lay)
        else:
            lay.experts, lay.shared = [], []
            host_layers.append(lay)
    setup_s = time.time() - t0

    def inputs_for(li, T):
        lay = host_layers[li]
        x = to_dev(lay.x[:T])
        lg = None if lay.logits is None else to_dev(lay.logits[:T])
        return x, lg

    def run_phase(T, steps, warmup):
        xs = [inputs_for(li, T) for li in range(n_layers)]
        stream = torch.cuda.current_stream()

        def one_step(i):
            if args.workload == "stress":
                for li in range(n_layers):
                    layers[li].forward(xs[li][0], xs[li][1])
            else:
                li = i % n_layers
                layers[li].forward(xs[li][0], xs[li][1])

        for i in range(max(warmup, n_layers)):
            one_step(i)
        torch.cuda.synchronize()
        timed_step = one_step
        if not args.no_graph:
            # the step is a fixed sequence of kernel launches: capture it once per weight set
            graphs = []
            for v in range(1 if args.workload == "stress" else n_layers):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    one_step(v)
                graphs.append(g)
            timed_step = lambda i: graphs[i % len(graphs)].replay()
            for i in range(warmup):
                timed_step(i)
            torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record(stream)
        for i in range(steps):
            timed_step(i)
        ev1.record(stream)
        torch.cuda.synchronize()
        ms_step = ev0.elapsed_time(ev1) / steps
        # second pass: HIP events around the gate/up kernel of the routed-expert FFN call
        calls_per_step = (n_layers if args.workload == "stress" else 1) * (2 if Fs else 1)
        for l in layers:                 # kernels one after the other, so that each probe pair times one kernel alone
            l.overlap_shared = l.merge_shared = False
        hm.hmoe_probe_arm(steps * calls_per_step)
        for i in range(steps):
            one_step(i)
        torch.cuda.synchronize()
        ms = hm.hmoe_probe_read(steps * calls_per_step)
        for l in layers:
            l.overlap_shared = l.merge_shared = l.fused
        routed_ms = ms[0::2] if Fs else ms        # routed call first, shared call second
        shared_ms = ms[1::2] if Fs else np.zeros(0, np.float32)
        # what the routed gate/up kernel touched (distinct experts with rows, last step's routing)
        used = range(n_layers) if args.workload == "stress" else range(min(n_layers, steps))
        distinct = float(np.mean([(np.diff(layers[li].offsets.cpu().numpy()) > 0).sum() for li in used]))
        return ms_step, float(np.mean(routed_ms)), float(np.mean(shared_ms)) if shared_ms.size else 0.0, distinct

    results = {}
    for name, T in phases:
        steps = args.steps
        ms_step, gu_ms, gu_shared_ms, distinct = run_phase(T, steps, args.warmup)
        A = T * K
        tokens = T * (n_layers if args.workload == "stress" else 1)
        # algorithmic work of the routed gate/up kernel: 2 of an expert's 3 matrices per distinct
        # touched expert + activations in/out; 4*H*F flops per assignment
        gu_bytes = distinct * 2 * H * F * w_bytes + A * H * elem + A * F * elem
        gu_flops = 4.0 * H * F * A
        hbm_frac = gu_bytes / (gu_ms * 1e-3) / 1e9 / HBM_PEAK_GBS
        mfma_frac = gu_flops / (gu_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS
        layer_bytes = distinct * 3 * H * F * w_bytes + (3 * H * Fs * w_bytes if Fs else 0)
        layer_flops = 6.0 * H * F * A + 6.0 * H * Fs * T
        per_layer_ms = ms_step / (n_layers if args.workload == "stress" else 1)
        results[name] = {
            "tokens": T, "ms_per_step": ms_step, "tokens_per_s": tokens / (ms_step * 1e-3),
            "distinct_experts": distinct,
            "gate_up_kernel_ms": gu_ms, "gate_up_GBps": gu_bytes / (gu_ms * 1e-3) / 1e9,
            "gate_up_TFLOPs": gu_flops / (gu_ms * 1e-3) / 1e12,
            "gate_up_hbm_frac": hbm_frac, "gate_up_mfma_frac": mfma_frac,
            "shared_gate_up_kernel_ms": gu_shared_ms,
            "layer_GBps": layer_bytes / (per_layer_ms * 1e-3) / 1e9,
            "layer_TFLOPs": layer_flops / (per_layer_ms * 1e-3) / 1e12,
            "layer_hbm_frac": layer_bytes / (per_layer_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "layer_mfma_frac": layer_flops / (per_layer_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        }

    main_name, main_T = phases[-1]
    main = results[main_name]
    if main["gate_up_mfma_frac"] >= main["gate_up_hbm_frac"]:
        roofline = {"bound": "mfma", "achieved": main["gate_up_TFLOPs"], "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": main["gate_up_mfma_frac"], "traffic": None}
    else:
        roofline = {"bound": "hbm", "achieved": main["gate_up_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": main["gate_up_hbm_frac"], "traffic": None}
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(traffic_file):   # HBM bytes per launch from rocprofv3 FETCH_SIZE + WRITE_SIZE runs (see profiles/)
        with open(traffic_file) as fh:
            roofline["traffic"] = json.load(fh).get("%s/%s%s" % (args.workload, main_name, "+w4" if w4 else ""))
    roofline["kernel"] = "ffn gate/up (routed experts), phase " + main_name
    roofline["kernel_ms"] = main["gate_up_kernel_ms"]

    # ---- staging: the workload's real cache size, misses copied from pinned host memory --------
    staging = None
    if not args.no_staging and shape.n_slots < E and args.workload != "stress":
        lay0 = host_layers[0]
        d2 = hm.make_desc(H, F, E, K, shape.n_slots, dtype_id)
        for l in layers[1:]:
            l.close()
        part = hm.MoELayer(d2, lay0.experts, lay0.shared, lay0.w_router, max_tokens=max_T)
        staging = {}
        for name, T in phases:
            n_steps = 8
            xs = []
            for i in range(n_steps + 1):
                xi = wl.make_x(shape, 777 + i, T)
                lgi = wl.make_logits(shape, 777 + i, T)
                xs.append((to_dev(xi), None if lgi is None else to_dev(lgi)))
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
            staging[name] = {"tokens_per_s_incl_pcie": T * n_steps / dt, "ms_per_step": dt / n_steps * 1e3,
                             "hit_rate": hits / max(1, needed), "staged_GB_per_step": part.staged_bytes / n_steps / 1e9,
                             "pcie_GBps_lower_bound": part.staged_bytes / dt / 1e9}
        # replacement policies on consecutive decode steps with temporal locality (Section IV-D, Fig. 8):
        # the same logit sequence served under LRU and under the score-aware policy of Eq. (3)
        policies = {}
        name, T = phases[0]
        if "decode" in name:
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
            staging[name]["hit_rate_correlated_steps"] = dict(policies, steps=n_seq - n_skip, rho=0.9, alpha=0.5)
        part.close()

    # ---- CPU baseline: the oracle as it stands, bounded sample -------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import moe_oracle as orc
        lay0 = host_layers[0]
        sample = min(main_T, {"toy": 16, "mixtral": 512, "dsv2lite": 1024, "qwen2moe": 256, "stress": 512}[args.workload])
        sub = np.arange(sample) * (main_T // sample)
        if lay0.logits is None:
            logits = orc.router_logits(wl.as_f64(lay0.x[:main_T]), wl.as_f64(lay0.w_router))
        else:
            logits = lay0.logits[:main_T]
        decode_weights = wl.as_f64
        if w4:      # the oracle's own quantiser: every weight replaced by the value its 4-bit code stands for
            from oracle import w4_oracle
            decode_weights = lambda m: w4_oracle.dequantize_w4(*w4_oracle.quantize_w4(wl.as_f32(m)))
        t1 = time.time()
        reps = 0
        while True:                       # repeat until about 10 s of host work have been timed
            orc.moe_layer(wl.as_f64(lay0.x[:main_T]), logits, K, lay0.experts, lay0.shared, token_subset=sub,
                          to_f64=decode_weights)
            reps += 1
            dt = time.time() - t1
            if dt >= 10.0 or reps >= 50:
                break
        cpu = {"value": sample * reps / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
               "sample": "%d of the %d %s tokens (every %d-th), full layer in float64 numpy, %d repetitions in %.1f s"
                         % (sample, main_T, main_name, main_T // sample, reps, dt)}

    out = {
        "metric": "MoE-layer tokens/s", "value": main["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": main["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": ("bf16 (4-bit weights)" if w4 else "bf16") if bf16 else "f32", "data": "synthetic",
        "config": {"workload": "%s/%s%s" % (args.workload, main_name, "+w4" if w4 else ""), "hidden": H, "ffn": F, "experts": E, "top_k": K,
                   "shared_ffn": list(shape.shared_ffn), "tokens": main_T, "layers": n_layers, "launch": "eager" if args.no_graph else "hip-graph replay",
                   "resident": "all needed experts resident in HBM slots (staging reported separately)"},
        "roofline": roofline, "cpu_baseline": cpu, "phases": results, "staging": staging, "setup_s": setup_s,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
