"""Pins for the CPU oracle: each check ties a part of oracle/moe_oracle.py to
something other than itself (closed forms, brute force, invariants, textbook
special cases), so that a dropped term, a wrong sign or index, or a transposed
operand fails at least one of them.  No GPU."""
import math
import os
from collections import OrderedDict

import numpy as np
import pytest

import workloads as wl
from oracle import moe_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = np.array([float(v) for v in vals], dtype=np.float64)
    return out


# ----------------------------------------------------------------------------- TopK
def test_topk_matches_full_stable_argsort():
    rng = np.random.default_rng(1)
    for n_experts, k in [(8, 2), (64, 6), (64, 8), (5, 5), (100, 7)]:
        lg = rng.standard_normal((200, n_experts)).astype(np.float32)
        lg[::3] = np.round(lg[::3] * 2) / 2       # many exact duplicates
        idx, _ = orc.route(lg, k)
        for t in range(lg.shape[0]):
            full = sorted(range(n_experts), key=lambda e: (-float(lg[t, e]), e))
            assert idx[t].tolist() == full[:k]


def test_topk_hand_cases():
    idx, w = orc.route(np.zeros((1, 8), np.float32), 3)          # all equal -> lowest indices
    assert idx.tolist() == [[0, 1, 2]]
    np.testing.assert_allclose(w, 1.0 / 3.0, rtol=1e-7)
    idx, _ = orc.route(np.arange(8, dtype=np.float32)[None], 3)   # strictly increasing
    assert idx.tolist() == [[7, 6, 5]]
    # duplicates straddling the k-th place: values 5 at {1, 4, 6}, k = 2 -> 1 then 4
    idx, _ = orc.route(np.array([[0, 5, 1, 2, 5, 3, 5, 4]], np.float32), 2)
    assert idx.tolist() == [[1, 4]]
    # +0.0 and -0.0 compare equal: index decides
    idx, _ = orc.route(np.array([[-0.0, 0.0, -1.0, 0.0]], np.float32), 2)
    assert idx.tolist() == [[0, 1]]


# ----------------------------------------------------------------------------- gate weights
def test_gate_closed_forms():
    # logits = ln([1, 4, 2, 3]); top-2 keeps experts 1 and 3 with weights 4/7 and 3/7
    lg = np.log(np.array([[1.0, 4.0, 2.0, 3.0]])).astype(np.float32)
    idx, w = orc.route(lg, 2)
    assert idx.tolist() == [[1, 3]]
    np.testing.assert_allclose(w[0], [4 / 7, 3 / 7], rtol=2e-7)
    # k = 1 -> weight exactly 1
    _, w1 = orc.route(lg, 1)
    assert w1.tolist() == [[1.0]]


def test_gate_sums_to_one_and_k_equals_e_is_softmax():
    rng = np.random.default_rng(2)
    lg = (rng.standard_normal((64, 16)) * 3).astype(np.float32)
    _, w = orc.route(lg, 4)
    np.testing.assert_allclose(w.astype(np.float64).sum(axis=1), 1.0, atol=1e-6)
    idx, wfull = orc.route(lg, 16)
    ref = np.exp(lg.astype(np.float64))
    ref /= ref.sum(axis=1, keepdims=True)
    np.testing.assert_allclose(wfull, np.take_along_axis(ref, idx.astype(np.int64), axis=1), rtol=1e-6)


def test_gate_equals_full_softmax_renormalised_over_topk():
    rng = np.random.default_rng(3)
    lg = rng.standard_normal((50, 64)).astype(np.float32)
    idx, w = orc.route(lg, 6)
    p = np.exp(lg.astype(np.float64) - lg.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    sel = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    np.testing.assert_allclose(w, sel / sel.sum(axis=1, keepdims=True), rtol=1e-6)


# ----------------------------------------------------------------------------- permutation
def _brute_permute(keys, n_experts):
    perm = []
    offsets = [0]
    for e in range(n_experts):
        for a, key in enumerate(keys):
            if key == e:
                perm.append(a)
        offsets.append(len(perm))
    return offsets, perm


def test_permute_invariants_and_brute_force():
    rng = np.random.default_rng(4)
    for n_tokens, n_experts, k in [(1, 8, 2), (16, 8, 2), (257, 64, 6), (0, 8, 2), (33, 5, 5)]:
        idx = np.stack([rng.permutation(n_experts)[:k] for _ in range(n_tokens)]).astype(np.int32) \
            if n_tokens else np.zeros((0, k), np.int32)
        offsets, perm, inv = orc.permute(idx, n_experts)
        n_assign = n_tokens * k
        keys = idx.reshape(-1)
        assert sorted(perm.tolist()) == list(range(n_assign))
        assert np.array_equal(inv[perm], np.arange(n_assign))
        assert np.all(np.diff(keys[perm]) >= 0)
        for e in range(n_experts):
            seg = perm[offsets[e]:offsets[e + 1]]
            assert np.all(np.diff(seg) > 0)                      # stable: ascending within a key
            assert np.all(keys[seg] == e)
        assert np.array_equal(np.diff(offsets), np.bincount(keys, minlength=n_experts))
        bo, bp = _brute_permute(keys.tolist(), n_experts)
        assert offsets.tolist() == bo and perm.tolist() == bp


def test_gather_then_scatter_is_identity():
    rng = np.random.default_rng(5)
    k, n_tokens = 3, 20
    idx = np.stack([rng.permutation(8)[:k] for _ in range(n_tokens)]).astype(np.int32)
    _, perm, inv = orc.permute(idx, 8)
    x = rng.standard_normal((n_tokens, 7))
    xp = orc.gather_rows(x, perm, k)
    for t in range(n_tokens):
        for j in range(k):
            assert np.array_equal(xp[inv[t * k + j]], x[t])


# ----------------------------------------------------------------------------- expert FFN
def test_swiglu_hand_case():
    g = _read_golden("swiglu_hand_case.txt")
    o = orc.expert_ffn(g["x"][None], g["w_gate"].reshape(3, 2), g["w_up"].reshape(3, 2),
                       g["w_down"].reshape(2, 3))
    np.testing.assert_allclose(o[0], g["o"], rtol=1e-13)


def test_ffn_special_cases():
    rng = np.random.default_rng(6)
    hid, ffn = 12, 12
    x = rng.standard_normal((5, hid))
    wg = rng.standard_normal((ffn, hid))
    wu = rng.standard_normal((ffn, hid))
    wd = rng.standard_normal((hid, ffn))
    assert np.all(orc.expert_ffn(x, np.zeros_like(wg), wu, wd) == 0)      # silu(0) = 0
    # W_up picks coordinate f of x, W_down = I  ->  o = silu(W_gate x) * x
    o = orc.expert_ffn(x, wg, np.eye(hid), np.eye(hid))
    gz = x @ wg.T
    np.testing.assert_allclose(o, gz / (1 + np.exp(-gz)) * x, rtol=1e-12)
    # linear in W_down
    np.testing.assert_allclose(orc.expert_ffn(x, wg, wu, 3.0 * wd), 3.0 * orc.expert_ffn(x, wg, wu, wd), rtol=1e-12)
    # large |g|: silu(g) -> g for g >> 0 and -> 0 for g << 0
    big = orc.expert_ffn(np.array([[40.0]]), np.array([[1.0], [-1.0]]), np.ones((2, 1)), np.eye(2))
    np.testing.assert_allclose(big[0], [40.0 * 40.0, -40.0 * math.exp(-40.0) / (1 + math.exp(-40.0)) * 40.0], rtol=1e-12)


# ----------------------------------------------------------------------------- whole layer
@pytest.mark.parametrize("n_experts,k,n_shared", [(8, 2, 0), (6, 3, 2), (4, 1, 1), (4, 4, 0)])
def test_layer_equals_dense_masked_brute_force(n_experts, k, n_shared):
    shape = wl.small_shape(hidden=24, ffn=40, n_experts=n_experts, top_k=k, shared_ffn=(16,) * n_shared)
    lay = wl.make_layer(shape, seed=11 + n_experts, n_tokens=9)
    logits = orc.router_logits(lay.x, lay.w_router)
    y = orc.moe_layer(lay.x, logits, k, lay.experts, lay.shared)
    yb = orc.dense_masked(lay.x, logits, k, lay.experts, lay.shared)
    np.testing.assert_allclose(y, yb, rtol=1e-10, atol=1e-12)
    assert np.abs(yb).max() > 1e-3          # the case is not vacuous


def test_toy_config_equals_dense_masked():
    """Workload 1 (16 tokens, hidden 256, 8 experts, FFN 512, top-2, seed 0), 4 of its tokens."""
    lay = wl.make_layer(wl.TOY, seed=0, n_tokens=16)
    logits = orc.router_logits(lay.x, lay.w_router)
    y = orc.moe_layer(lay.x, logits, 2, lay.experts)
    sub = [0, 5, 10, 15]
    yb = orc.dense_masked(lay.x[sub], logits[sub], 2, lay.experts)
    np.testing.assert_allclose(y[sub], yb, rtol=1e-9, atol=1e-15)


def test_layer_token_independence_and_subset():
    shape = wl.small_shape(hidden=16, ffn=24, n_experts=8, top_k=2, shared_ffn=(8,))
    lay = wl.make_layer(shape, seed=3, n_tokens=12)
    logits = orc.router_logits(lay.x, lay.w_router)
    y = orc.moe_layer(lay.x, logits, 2, lay.experts, lay.shared)
    sub = np.array([7, 2, 11])
    ys = orc.moe_layer(lay.x, logits, 2, lay.experts, lay.shared, token_subset=sub)
    np.testing.assert_allclose(ys, y[sub], rtol=1e-12)


def test_two_shared_experts_equal_one_concatenated():
    shape = wl.small_shape(hidden=16, ffn=24, n_experts=4, top_k=2, shared_ffn=(8, 8))
    lay = wl.make_layer(shape, seed=5, n_tokens=6)
    logits = orc.router_logits(lay.x, lay.w_router)
    y2 = orc.moe_layer(lay.x, logits, 2, lay.experts, lay.shared)
    (g0, u0, d0), (g1, u1, d1) = lay.shared
    cat = (np.concatenate([g0, g1]), np.concatenate([u0, u1]), np.concatenate([d0, d1], axis=1))
    y1 = orc.moe_layer(lay.x, logits, 2, lay.experts, [cat])
    np.testing.assert_allclose(y1, y2, rtol=1e-12)


def test_router_logits_orientation():
    x = np.array([[1.0, 2.0, 3.0]])
    wg = np.array([[1.0, 0.0, 0.0], [0.0, 0.0, 2.0]])            # [E, H]
    assert orc.router_logits(x, wg).tolist() == [[1.0, 6.0]]


# ----------------------------------------------------------------------------- expert cache
def test_cache_hand_trace_single_requests():
    c = orc.ExpertCacheModel(n_experts=4, n_slots=2)
    got = [c.serve([e]) for e in (0, 1, 2, 0, 3)]
    assert got == [[(0, 0, 0, -1)], [(1, 1, 0, -1)], [(2, 0, 1, 0)], [(0, 1, 1, 1)], [(3, 0, 1, 2)]]
    assert c.expert_in == [3, 0] and c.slot_of == [1, -1, -1, 0]


def test_cache_hand_trace_waves():
    c = orc.ExpertCacheModel(n_experts=8, n_slots=2)
    plan = c.serve([0, 1, 2, 3, 4, 5])
    assert plan == [(0, 0, 0, -1), (1, 1, 0, -1), (2, 0, 1, 0), (3, 1, 1, 1), (4, 0, 2, 2), (5, 1, 2, 3)]
    c = orc.ExpertCacheModel(n_experts=8, n_slots=4)
    assert c.serve([5, 0, 1]) == [(0, 0, 0, -1), (1, 1, 0, -1), (5, 2, 1, 2)]
    # mixtral-like: 4 slots, 7 of 8 experts needed -> three misses, all in wave 1, slots 0, 1, 2
    c = orc.ExpertCacheModel(n_experts=8, n_slots=4)
    plan = c.serve([0, 1, 2, 3, 4, 5, 6])
    assert plan[4:] == [(4, 0, 1, 0), (5, 1, 1, 1), (6, 2, 1, 2)]


def test_cache_matches_textbook_lru_and_invariants():
    rng = np.random.default_rng(7)
    n_experts, n_slots = 16, 5
    c = orc.ExpertCacheModel(n_experts, n_slots)
    lru = OrderedDict((e, None) for e in range(n_slots))       # textbook LRU, oldest first
    for _ in range(500):
        e = int(rng.integers(n_experts))
        hit_model = c.slot_of[e] >= 0
        hit_ref = e in lru
        assert hit_model == hit_ref
        if hit_ref:
            lru.move_to_end(e)
        else:
            if len(lru) == n_slots:
                lru.popitem(last=False)
            lru[e] = None
        c.serve([e])
        assert sorted(x for x in c.expert_in if x >= 0) == sorted(lru)
        for ex in range(n_experts):                            # mutually inverse partial maps
            if c.slot_of[ex] >= 0:
                assert c.expert_in[c.slot_of[ex]] == ex
        assert sum(s >= 0 for s in c.slot_of) <= n_slots


def test_cache_multi_expert_calls_every_needed_expert_served_once():
    rng = np.random.default_rng(8)
    c = orc.ExpertCacheModel(12, 4)
    for _ in range(200):
        need = rng.choice(12, size=int(rng.integers(1, 10)), replace=False).tolist()
        plan = c.serve(need)
        assert sorted(p[0] for p in plan) == sorted(need)
        by_wave = {}
        for e, s, w, v in plan:
            by_wave.setdefault(w, []).append(s)
        for w, slots in by_wave.items():
            assert len(set(slots)) == len(slots)               # one expert per slot in a wave
        waves = {e: w for e, _, w, _ in plan}
        for e, s, w, v in plan:
            if v in waves:
                assert w == waves[v] + 1                       # never overwrite before the victim ran


def test_cache_evict_hand_trace():
    """Dropping an expert frees its slot; the next miss takes the lowest-numbered free slot before any
    occupant is replaced, and an expert that is not resident is dropped without effect (traced by hand)."""
    c = orc.ExpertCacheModel(n_experts=4, n_slots=2)
    c.serve([0])                                   # tick[0] = 1
    c.serve([1])                                   # tick[1] = 2
    c.evict(0)
    assert c.slot_of == [-1, 1, -1, -1] and c.expert_in == [-1, 1]
    c.evict(3)                                     # not resident: nothing changes
    assert c.slot_of == [-1, 1, -1, -1] and c.expert_in == [-1, 1]
    assert c.serve([2]) == [(2, 0, 1, -1)]         # the free slot, nobody replaced; tick[2] = 4
    assert c.serve([3]) == [(3, 1, 1, 1)]          # no free slot: expert 1 (tick 2) is older than expert 2 (tick 4)
    c.evict(3)
    c.evict(2)
    assert c.slot_of == [-1, -1, -1, -1] and c.expert_in == [-1, -1]
    assert c.serve([1, 0]) == [(0, 0, 1, -1), (1, 1, 1, -1)]   # misses in ascending id, lowest free slot each
    assert c.slot_of == [0, 1, -1, -1]


def test_cache_evict_keeps_the_maps_inverse():
    rng = np.random.default_rng(11)
    c = orc.ExpertCacheModel(10, 4)
    for _ in range(300):
        if rng.random() < 0.3:
            e = int(rng.integers(10))
            was = c.slot_of[e]
            c.evict(e)
            assert c.slot_of[e] == -1 and (was < 0 or c.expert_in[was] == -1)
        else:
            need = rng.choice(10, size=int(rng.integers(1, 5)), replace=False).tolist()
            free_before = [s for s in range(4) if c.expert_in[s] < 0]
            plan = c.serve(need)
            misses = [p for p in plan if p[2] > 0]
            for (e, s, w, v), want in zip(misses, free_before):   # free slots go first, lowest first, nobody replaced
                assert s == want and v == -1
        for ex in range(10):
            if c.slot_of[ex] >= 0:
                assert c.expert_in[c.slot_of[ex]] == ex
        for s in range(4):
            if c.expert_in[s] >= 0:
                assert c.slot_of[c.expert_in[s]] == s


# ----------------------------------------------------------------------------- input recipe
def test_bf16_rounding_is_nearest_even():
    a = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e-5], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    got = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(a))
    assert got[0] == 1.0 and got[1] == 1.0 and got[2] == 1.015625 and got[3] == -2.5
    assert abs(got[4] - a[4]) <= abs(a[4]) * 2.0 ** -8


def test_workload_recipes():
    lg = wl.make_logits(wl.QWEN2MOE, 3, 40)
    assert np.all(np.argmax(lg[::10], axis=1) == 0)
    b = wl.zipf_bias(64)
    assert b[0] > b[1] > b[63] and abs(np.exp(b.astype(np.float64)).sum() / 64 - 1.0) < 1e-6
    x = wl.as_f64(wl.make_x(wl.MIXTRAL, 1, 4))
    np.testing.assert_allclose((x ** 2).mean(axis=1), 1.0, rtol=2e-2)
    lay_a = wl.make_layer(wl.small_shape(), 9, 4)
    lay_b = wl.make_layer(wl.small_shape(), 9, 4)
    assert np.array_equal(lay_a.experts[3][2], lay_b.experts[3][2])
    # decode-step sequences: stationary N(0,1) per step, lag-1 correlation rho, the workload's forcing at every step
    seq = wl.make_logit_sequence(wl.small_shape(n_experts=8), 4, 16, 400, 0.9)
    assert seq.shape == (400, 16, 8) and seq.dtype == np.float32
    assert abs(seq.std() - 1.0) < 0.05 and abs(seq[300:].std() - seq[:100].std()) < 0.1
    lag1 = np.mean(seq[:-1] * seq[1:]) / np.mean(seq * seq)
    assert abs(lag1 - 0.9) < 0.03
    indep = wl.make_logit_sequence(wl.small_shape(n_experts=8), 4, 16, 400, 0.0)
    assert abs(np.mean(indep[:-1] * indep[1:])) < 0.02
    hot = wl.make_logit_sequence(wl.QWEN2MOE, 3, 20, 5, 0.9)
    assert np.all(np.argmax(hot[:, ::10], axis=2) == 0)


# ----------------------------------------------------------------------------- score-aware replacement, Eq. (3)
def test_mrs_update_hand_values_and_closed_form():
    # alpha = 0.5, p = 2: only the two largest scores are accumulated
    s1 = [0.1, 0.5, 0.3, 0.1]
    S = orc.mrs_update([0.0] * 4, s1, 0.5, 2)
    assert S == [0.0, 0.25, 0.15, 0.0]
    S = orc.mrs_update(S, [0.6, 0.1, 0.2, 0.1], 0.5, 2)
    np.testing.assert_allclose(S, [0.3, 0.125, 0.175, 0.0], rtol=1e-15)
    # ties at the p-th place: lower id is kept
    assert orc.mrs_update([0.0] * 3, [0.2, 0.2, 0.2], 1.0, 2) == [0.2, 0.2, 0.0]
    # constant scores: S_n = s * (1 - (1 - alpha)^n)
    S = [0.0, 0.0]
    for n in range(1, 8):
        S = orc.mrs_update(S, [0.7, 0.3], 0.3, 2)
        np.testing.assert_allclose(S, [0.7 * (1 - 0.7 ** n), 0.3 * (1 - 0.7 ** n)], rtol=1e-12)


def test_route_scores_is_mean_softmax():
    lg = np.log(np.array([[1.0, 1.0, 2.0], [3.0, 1.0, 0.0 + 1e-300]]))
    lg[1, 2] = -745.0          # exp underflows to 0
    np.testing.assert_allclose(orc.route_scores(lg), [(0.25 + 0.75) / 2, (0.25 + 0.25) / 2, 0.25], rtol=1e-12)


def test_mrs_cache_evicts_lowest_score_and_keeps_wave_order():
    c = orc.MRSCacheModel(n_experts=6, n_slots=3, alpha=1.0)
    c.update([0.05, 0.4, 0.3, 0.1, 0.1, 0.05], top_p=6)       # S = s
    assert c.serve([3]) == [(3, 0, 1, 0)]                      # resident 0,1,2: expert 0 has the lowest S
    assert c.serve([4]) == [(4, 0, 1, 3)]                      # now 3 (0.1) < 2 (0.3) < 1 (0.4)
    # all residents needed: they form wave 0 and are evicted in order of S; misses run one wave later
    c = orc.MRSCacheModel(n_experts=6, n_slots=2, alpha=1.0)
    c.update([0.3, 0.1, 0.2, 0.2, 0.1, 0.1], top_p=6)
    assert c.serve([0, 1, 2, 3]) == [(0, 0, 0, -1), (1, 1, 0, -1), (2, 1, 1, 1), (3, 0, 1, 0)]
    # invariants under random use
    rng = np.random.default_rng(0)
    c = orc.MRSCacheModel(10, 4, 0.4)
    for _ in range(200):
        need = rng.choice(10, size=int(rng.integers(1, 8)), replace=False).tolist()
        plan = c.serve(need)
        assert sorted(p[0] for p in plan) == sorted(need)
        c.update(rng.random(10), 4)
        for ex in range(10):
            if c.slot_of[ex] >= 0:
                assert c.expert_in[c.slot_of[ex]] == ex
