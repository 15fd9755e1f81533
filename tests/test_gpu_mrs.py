"""Score-aware (Minus Recent Score, Section IV-D, Eq. (3)) replacement: the routing-score kernel and
the library's victim choice against the oracle's MRS cache model, over a sequence of decode steps."""
import sys

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe_oracle as orc
from hmoe_testlib import TOL, build_layer, max_rel_err, oracle_layer, to_device, to_host_f32

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def hm():
    import paper_2504_05897_amd as hm
    return hm


@pytest.mark.parametrize("T,E", [(1, 8), (7, 64), (300, 64), (5000, 60), (257, 200)])
def test_route_scores(hm, T, E):
    print("route_scores", T, E, flush=True)
    rng = np.random.default_rng(T + E)
    lg = (rng.standard_normal((T, E)) * 2).astype(np.float32)
    d = hm.make_desc(64, 64, E, 1, E, hm.HMOE_BF16)
    scores = torch.zeros(E, dtype=torch.float32, device=DEV)
    host = torch.zeros(E, dtype=torch.float32, pin_memory=True)
    ws_bytes = hm.hmoe_route_scores_workspace_bytes(d, T)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    got = []
    for _ in range(2):                       # fixed summation order: identical bits on every run
        hm.hmoe_route_scores(d, to_device(lg), T, scores, host, ws, ws_bytes)
        torch.cuda.synchronize()
        got.append(host.numpy().copy())
    assert np.array_equal(got[0], got[1]) and np.array_equal(got[0], scores.cpu().numpy())
    ref = orc.route_scores(lg)
    np.testing.assert_allclose(got[0], ref, rtol=2e-5, atol=1e-8)
    assert abs(got[0].astype(np.float64).sum() - 1.0) < 1e-5


def test_mrs_slot_maps_follow_the_oracle(hm):
    """4 slots, 8 experts, temporally correlated logits: after every step the slot map, the plan and the
    priority estimates S equal the oracle's MRS model fed with the same routing scores."""
    print("mrs sequence", flush=True)
    shape = wl.small_shape(dtype=wl.BF16, hidden=64, ffn=64, n_experts=8, top_k=2, n_slots=4, x_mode="rmsnorm")
    base = wl.make_layer(shape, 2, 1)
    layer = build_layer(hm, base, max_tokens=8)
    alpha = 0.25          # exactly representable: the ABI takes alpha as a float
    layer.set_policy(hm.HMOE_POLICY_MRS, alpha)
    model = orc.MRSCacheModel(8, 4, alpha)
    rng = np.random.default_rng(5)
    prev = rng.standard_normal((8, 8)).astype(np.float32)
    evicted_not_lru = 0
    for step in range(24):
        T = [1, 2, 1, 8, 1, 3][step % 6]
        prev = (0.8 * prev + 0.6 * rng.standard_normal((8, 8))).astype(np.float32)    # AR(1) logits
        logits = np.ascontiguousarray(prev[:T])
        lay = wl.make_layer(shape, 900 + step, T, with_weights=False)
        lay.experts, lay.shared = base.experts, base.shared
        lg_dev = to_device(logits)
        y = layer.forward(to_device(lay.x), lg_dev)
        torch.cuda.synchronize()
        ridx, _ = orc.route(logits, 2)
        plan = model.serve(np.unique(ridx).tolist())
        assert layer.slot_map() == model.slot_of, (step, plan)
        wave, slot, victim, n_waves = layer.last_plan
        for (e, s, w, v) in plan:
            assert wave[e] == w and slot[e] == s and victim[e] == v
        err = max_rel_err(to_host_f32(y), oracle_layer(lay, logits))
        assert err < TOL[wl.BF16]
        s_used = layer.update_scores(lg_dev)
        np.testing.assert_allclose(s_used, orc.route_scores(logits), rtol=2e-5, atol=1e-8)
        model.update(s_used, 4)
        np.testing.assert_array_equal(hm.hmoe_cache_get_scores(layer.cache, 8), np.array(model.score))
    layer.close()


def test_policy_arguments(hm):
    shape = wl.small_shape(dtype=wl.BF16, hidden=64, ffn=64, n_experts=4, top_k=2, n_slots=2)
    layer = build_layer(hm, wl.make_layer(shape, 1, 1), max_tokens=2)
    for bad in [(7, 0.5), (hm.HMOE_POLICY_MRS, 0.0), (hm.HMOE_POLICY_MRS, 1.5)]:
        with pytest.raises(hm.HmoeError) as ei:
            hm.hmoe_cache_set_policy(layer.cache, *bad)
        assert ei.value.status == hm.HMOE_ERR_INVALID_ARG
    hm.hmoe_cache_set_policy(layer.cache, hm.HMOE_POLICY_MRS, 1.0)
    hm.hmoe_cache_update_scores(layer.cache, np.array([0.1, 0.2, 0.3, 0.4], np.float32), 2)
    assert hm.hmoe_cache_get_scores(layer.cache, 4).tolist() == [0.0, 0.0, float(np.float32(0.3)), float(np.float32(0.4))]
    layer.close()
