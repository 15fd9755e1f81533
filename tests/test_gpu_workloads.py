"""Parity at the full sizes of the five workloads, in the launch configuration the benchmark
times (AUTO kernel choice, fused front end, real cache sizes with staging from pinned host memory).

Integer results (top-k ids, offsets, permutation, slot map) are compared in full and bit for bit.
The layer output is compared on every token for small batches and on a stratified sample of at least
256 tokens for prefill batches (tokens are independent in Eq. (1), so the oracle evaluates the sampled
ones one by one): for every expert with rows, the tokens behind the first and the last sorted row of its
first and of its last 128-row tile, then seeded random tokens up to the sample size.  The measure is
max|y - y_ref| / max|y_ref| over the compared tokens, 2e-2 for bf16 and 1e-4 for fp32.  Workloads whose
logits come from x . W_g run through the fused front end (forward(x, None)), as the benchmark does, and
once through the separate calls."""
import sys

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe_oracle as orc
from hmoe_testlib import TOL, build_layer, max_rel_err, oracle_layer, to_device, to_host_f32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hm():
    import paper_2504_05897_amd as hm
    return hm


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def stratified_tokens(offsets, perm, top_k, n_tokens, n_sample, seed, tile=128):
    """Tokens behind the first and last sorted row of the first and of the last `tile`-row tile of every expert
    with rows, plus seeded random tokens until there are at least n_sample (all tokens if n_sample >= n_tokens)."""
    if n_sample >= n_tokens:
        return np.arange(n_tokens)
    rows = []
    for e in range(len(offsets) - 1):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi > lo:
            last_tile = lo + (hi - 1 - lo) // tile * tile
            rows += [lo, min(lo + tile, hi) - 1, last_tile, hi - 1]
    picked = set(int(perm[p]) // top_k for p in rows)
    for t in np.random.default_rng(seed).permutation(n_tokens):
        if len(picked) >= n_sample:
            break
        picked.add(int(t))
    return np.array(sorted(picked))


def run_and_check(hm, layer, base, shape, seed, T, n_sample, model=None, fused_front=True):
    """One forward of `layer` on fresh seeded activations; returns the error on the sample."""
    lay = wl.make_layer(shape, seed, T, with_weights=False)
    lay.experts, lay.shared, lay.w_router = base.experts, base.shared, base.w_router
    x = to_device(lay.x)
    if lay.logits is None:
        ref_lg = orc.router_logits(wl.as_f64(lay.x), wl.as_f64(lay.w_router))
        if fused_front:      # router logits, routing and permutation through hmoe_router_route_permute, as benchmarked
            y = layer.forward(x, None)
        else:
            hm.hmoe_router_logits(layer.desc, x, layer.w_router, T, layer.logits)
            y = layer.forward(x, layer.logits[:T])
        logits = layer.logits[:T].cpu().numpy()
        assert np.abs(logits - ref_lg).max() <= 1e-5 * np.abs(ref_lg).max()
    else:
        logits = lay.logits
        y = layer.forward(x, to_device(logits))
    torch.cuda.synchronize()
    K, E = shape.top_k, shape.n_experts
    ridx, rw = orc.route(logits, K)
    ro, rp, ri = orc.permute(ridx, E)
    assert np.array_equal(layer.topk_idx[:T].cpu().numpy(), ridx)
    np.testing.assert_allclose(layer.topk_w[:T].cpu().numpy(), rw, rtol=2e-6, atol=1e-7)
    assert np.array_equal(layer.offsets.cpu().numpy(), ro)
    assert np.array_equal(layer.perm[:T * K].cpu().numpy(), rp)
    assert np.array_equal(layer.inv_perm[:T * K].cpu().numpy(), ri)
    if model is not None:
        plan = model.serve(np.unique(ridx).tolist())
        assert layer.slot_map() == model.slot_of
        assert np.array_equal(layer.slot_of.cpu().numpy(), np.array(model.slot_of, np.int32))
        wave = layer.last_plan[0]
        for (e, s, w, v) in plan:
            assert wave[e] == w
    sub = stratified_tokens(ro, rp, K, T, n_sample, seed)
    assert len(sub) >= min(T, n_sample)
    y_ref = oracle_layer(lay, logits, token_subset=sub)
    return max_rel_err(to_host_f32(y)[sub], y_ref)


def test_workload1_toy_fp32(hm):
    say("workload 1: toy fp32, seed 0")
    base = wl.make_layer(wl.TOY, 0, 16)
    layer = build_layer(hm, base)
    err = run_and_check(hm, layer, base, wl.TOY, 0, 16, 16)
    say("  err", err)
    layer.close()
    assert err < TOL[wl.F32]


def test_workload2_mixtral(hm):
    say("workload 2: mixtral, 4 of 8 experts cached")
    shape = wl.MIXTRAL
    base = wl.make_layer(shape, 1, 1, threads=16)
    layer = build_layer(hm, base, max_tokens=512)
    model = orc.ExpertCacheModel(shape.n_experts, shape.n_slots)
    for i, (T, n_sample) in enumerate([(1, 1), (1, 1), (8, 8), (1, 1), (512, 256), (8, 8)]):
        err = run_and_check(hm, layer, base, shape, 200 + i, T, n_sample, model, fused_front=i != 1)
        say("  T", T, "waves", layer.last_plan[3], "err", err)
        assert err < TOL[wl.BF16]
    layer.close()


def test_workload3_dsv2lite(hm):
    say("workload 3: deepseek-v2-lite style, Zipf logits, 32 of 64 experts cached")
    shape = wl.DSV2LITE
    base = wl.make_layer(shape, 2, 1, threads=16)
    layer = build_layer(hm, base, max_tokens=1024)
    model = orc.ExpertCacheModel(shape.n_experts, shape.n_slots)
    for i, (T, n_sample) in enumerate([(1, 1), (1, 1), (1024, 256), (1, 1)]):
        err = run_and_check(hm, layer, base, shape, 300 + i, T, n_sample, model)
        say("  T", T, "waves", layer.last_plan[3], "err", err)
        assert err < TOL[wl.BF16]
    layer.close()


def test_workload4_qwen2moe(hm):
    say("workload 4: qwen2-moe style, hot expert 0, 48 of 64 experts cached")
    shape = wl.QWEN2MOE
    base = wl.make_layer(shape, 3, 1, threads=16)
    layer = build_layer(hm, base, max_tokens=2048)
    model = orc.ExpertCacheModel(shape.n_experts, shape.n_slots)
    for i, (T, n_sample) in enumerate([(4, 4), (2048, 256), (4, 4)]):
        err = run_and_check(hm, layer, base, shape, 400 + i, T, n_sample, model)
        say("  T", T, "waves", layer.last_plan[3], "err", err)
        assert err < TOL[wl.BF16]
    layer.close()


def test_workload5_stress_layers(hm):
    say("workload 5: 16384 tokens, all experts resident, every one of the 27 stacked layers")
    from concurrent.futures import ThreadPoolExecutor
    shape = wl.STRESS
    with ThreadPoolExecutor(max_workers=1) as pool:      # the next layer's weights are drawn while this one is checked
        nxt = pool.submit(wl.make_layer, shape, 5000, 1, threads=12)
        for li in range(27):
            base = nxt.result()
            if li + 1 < 27:
                nxt = pool.submit(wl.make_layer, shape, 5000 + li + 1, 1, threads=12)
            layer = build_layer(hm, base, max_tokens=16384)
            err = run_and_check(hm, layer, base, shape, 5000 + li, 16384, 256, fused_front=li != 1)
            say("  layer", li, "err", err)
            layer.close()
            del layer, base
            assert err < TOL[wl.BF16]


def test_bench_line_contract():
    """bench.py prints one JSON line with the fields the harness reads: metric, value, timing, the roofline of the
    dominant kernel and the CPU-oracle baseline; the default run covers every bf16 workload and reports the largest
    (the MFMA-bound stress workload) as `value`; a GPU count above one is refused."""
    import json
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    print("bench contract", flush=True)
    # the default command with fewer stacked stress layers, so that the set-up stays short
    run = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--steps", "2", "--warmup", "1", "--blocks", "3",
                          "--layers", "2"], capture_output=True, text=True, timeout=600, cwd=root)
    assert run.returncode == 0, run.stderr[-2000:]
    lines = [l for l in run.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 2 and out["warmup"] == 1 and out["higher_is_better"] is True
    assert out["value"] > 0 and out["ms_per_step"] > 0 and out["config"]["workload"] == "stress/prefill16384"
    assert out["vs_baseline"] is None and out["dtype"] == "bf16"
    roof = out["roofline"]
    assert roof["bound"] == "mfma" and roof["unit"] == "TFLOP/s" and roof["peak"] == 2500.0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9 and 0 < roof["frac"] < 1
    assert roof["traffic"] is None or roof["traffic"] > 0
    cpu = out["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["value"] > 0 and cpu["cores"] >= 1 and cpu["unit"] == out["unit"] and cpu["sample"]
    want = ["mixtral/decode1", "mixtral/decode8", "mixtral/prefill512", "dsv2lite/decode1", "dsv2lite/prefill1024",
            "qwen2moe/decode4", "qwen2moe/prefill2048", "stress/prefill16384"]
    assert sorted(out["phases"]) == sorted(want)
    for name in want:
        ph = out["phases"][name]
        assert ph["ms_per_step_p10"] <= ph["ms_per_step"] <= ph["ms_per_step_p90"] and ph["blocks"] == 3
        for part in ("gate_up", "down", "layer"):
            assert ph[part]["bound"] in ("hbm", "mfma") and 0 < ph[part]["frac"] < 1.2, (name, part, ph[part])
    for name in ("dsv2lite/decode1", "qwen2moe/decode4"):   # decode steps of layers with shared experts: the merged launches
        for part in ("gate_up_with_shared", "down_with_shared"):
            assert 0 < out["phases"][name][part]["frac"] < 1.2, (name, part)
    assert out["value"] == out["phases"]["stress/prefill16384"]["tokens_per_s"]
    refused = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                             timeout=120, cwd=root)
    assert refused.returncode != 0 and "ONE GPU" in (refused.stderr + refused.stdout)
