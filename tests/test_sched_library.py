"""The library's host-side scheduling planner (Section IV-B) against the oracle: same plans, value for value, on
the hand-traced example and on random instances; error paths.  No GPU: the planner is host code."""
import numpy as np
import pytest

from oracle import sched_oracle as so


@pytest.fixture(scope="module")
def hm():
    import paper_2504_05897_amd as hm
    return hm


def rules_of(hm, flags):
    return ((hm.HMOE_SCHED_CPU_UNCACHED if flags["cpu_uncached"] else 0) | (hm.HMOE_SCHED_CPU_CACHED if flags["cpu_cached"] else 0)
            | (hm.HMOE_SCHED_TRANSFERS if flags["transfers"] else 0))


def same(got, plan):
    device, start, end, xfer, makespan = got[:5]
    assert device.tolist() == plan.device
    assert start.tolist() == plan.start and end.tolist() == plan.end and xfer.tolist() == plan.transfer_start
    assert makespan == plan.makespan


def test_hand_traced_example(hm):
    cost = hm.SchedCost(1, 0, 0, 1, 3)
    device, start, end, xfer, makespan = hm.hmoe_schedule_simulate([4, 2, 3, 1, 1], [1, 1, 0, 0, 1], cost)
    assert device.tolist() == [hm.HMOE_ON_GPU_CACHED, hm.HMOE_ON_GPU_CACHED, hm.HMOE_ON_GPU_LOADED, hm.HMOE_ON_CPU, hm.HMOE_ON_CPU]
    assert start.tolist() == [0, 1, 3, 0, 1] and end.tolist() == [1, 2, 4, 1, 2] and xfer.tolist() == [-1, -1, 0, -1, -1]
    assert makespan == 4


def test_random_instances_equal_the_oracle(hm):
    rng = np.random.default_rng(1)
    for trial in range(400):
        n = int(rng.integers(0, 40)) if trial % 10 else 256
        load = rng.integers(0, 12, n).tolist()
        cached = (rng.random(n) < rng.random()).tolist()
        vals = [float(v) for v in rng.choice([0.0, 0.25, 0.5, 1.0, 2.0, 3.0, 7.5], 5)]
        cost, ocost = hm.SchedCost(*vals), so.SchedCost(*vals)
        for flags in so.STRATEGIES:
            same(hm.hmoe_schedule_simulate(load, cached, cost, rules_of(hm, flags)), so.simulate(load, cached, ocost, **flags))
        got = hm.hmoe_schedule_plan(load, cached, cost)
        plan, which = so.hybrid_schedule(load, cached, ocost)
        same(got, plan)
        assert got[5] == rules_of(hm, so.STRATEGIES[which])


def test_errors(hm):
    cost = hm.SchedCost(1, 0, 0, 1, 3)
    with pytest.raises(hm.HmoeError) as ei:                       # nothing may compute the uncached expert
        hm.hmoe_schedule_simulate([1, 2], [1, 0], cost, hm.HMOE_SCHED_CPU_CACHED)
    assert ei.value.status == hm.HMOE_ERR_UNSUPPORTED
    for bad_load, bad_cost, rules in [([1, -2], cost, 7), ([1], hm.SchedCost(-1, 0, 0, 1, 3), 7), ([1], cost, 8),
                                      ([1], hm.SchedCost(1, 0, 0, float("nan"), 3), 7), ([1] * 257, cost, 7)]:
        with pytest.raises(hm.HmoeError) as ei:
            hm.hmoe_schedule_simulate(bad_load, [0] * len(bad_load), bad_cost, rules)
        assert ei.value.status == hm.HMOE_ERR_INVALID_ARG
    device, _, _, _, makespan, _ = hm.hmoe_schedule_plan([], [], cost)
    assert device.size == 0 and makespan == 0
