"""Pins for the oracle of the hybrid CPU-GPU scheduling simulation (Section IV-B).  The paper prints no numbers
for its worked example (they live in a figure), so the pins are: a schedule traced by hand from the three
priority rules under the cost model the example's text states (constant GPU time, CPU time equal to the load,
transfer of 3 units), which must show the outcome the figure's caption describes; closed forms; the
constraints a valid schedule obeys; a brute-force lower bound; the two fixed mappings as upper bounds."""
import itertools

import numpy as np
import pytest

from oracle import sched_oracle as so

GPU0, GPU1, CPU = so.ON_GPU_CACHED, so.ON_GPU_LOADED, so.ON_CPU


def test_hand_trace_with_the_outcome_of_the_papers_example():
    # experts A..E, loads 4 2 3 1 1; A, B, E cached; GPU 1 unit per expert, CPU = load, transfer 3.
    # GPU queue A(4) B(2) E(1); CPU queue D(1) C(3).
    # t=0: CPU takes D (ends 1); GPU takes A (ends 1); transfer takes C (arrives 3).
    # t=1: CPU has no uncached expert left -> takes the lowest cached one, E (ends 2); GPU takes B (ends 2).
    # t=2: only C is left, in flight: the GPU waits for it, computes it 3..4.  Makespan 4.
    # As in the caption of the paper's figure: the CPU computes cached expert E, the GPU the uncached C.
    cost = so.SchedCost(gpu_base=1, gpu_per_token=0, cpu_base=0, cpu_per_token=1, transfer=3)
    plan = so.simulate([4, 2, 3, 1, 1], [True, True, False, False, True], cost)
    assert plan.device == [GPU0, GPU0, GPU1, CPU, CPU]
    assert plan.start == [0, 1, 3, 0, 1] and plan.end == [1, 2, 4, 1, 2]
    assert plan.transfer_start == [-1, -1, 0, -1, -1] and plan.makespan == 4
    best, which = so.hybrid_schedule([4, 2, 3, 1, 1], [True, True, False, False, True], cost)
    assert which == 0 and best == plan
    # fixed mappings: uncached C, D on the CPU take 1 + 3 = 4 (a tie with the plan); loading both on demand
    # ends at 7 (C arrives at 3 and runs 3..4, D arrives at 6 and runs 6..7)
    assert so.fixed_mapping_makespan([4, 2, 3, 1, 1], [True, True, False, False, True], cost, True) == 4
    assert so.fixed_mapping_makespan([4, 2, 3, 1, 1], [True, True, False, False, True], cost, False) == 7


def test_hand_trace_slow_cpu_keeps_cached_experts_on_the_gpu():
    # three cached experts, CPU 10x the load: with the full rules the CPU grabs the lowest-load expert at t=0
    # and finishes at 10; without the take-over rule the GPU does all three by t=3.  The second strategy wins.
    cost = so.SchedCost(1, 0, 0, 10, 3)
    full = so.simulate([3, 2, 1], [True] * 3, cost)
    assert full.device == [GPU0, GPU0, CPU] and full.makespan == 10
    best, which = so.hybrid_schedule([3, 2, 1], [True] * 3, cost)
    assert which == 1 and best.device == [GPU0] * 3 and best.makespan == 3 and best.start == [0, 1, 2]


def test_ties_between_timelines_go_to_the_cpu_first():
    # one cached expert, everything free at t=0: under the full rules the CPU (named first) takes it
    cost = so.SchedCost(1, 0, 0, 1, 3)
    assert so.simulate([2], [True], cost).device == [CPU]
    best, which = so.hybrid_schedule([2], [True], cost)          # ... but the plan keeps it on the GPU: 1 < 2
    assert which == 1 and best.device == [GPU0] and best.makespan == 1
    # equal loads: lower id first in both queues
    p = so.simulate([2, 2, 2, 2], [True, True, False, False], cost, cpu_cached=False)
    assert p.start[0] < p.start[1] and p.device[2] == CPU and p.device[3] == GPU1


def test_closed_forms():
    cost = so.SchedCost(0.5, 0.25, 1.0, 2.0, 3.0)
    load = [5, 0, 2, 7, 1, 0, 3]
    n = len(load)
    # nothing activated
    p, _ = so.hybrid_schedule([0] * 4, [False] * 4, cost)
    assert p.makespan == 0 and p.device == [-1] * 4
    # all cached, CPU off: the GPU runs them back to back, highest load first
    p = so.simulate(load, [True] * n, cost, cpu_uncached=False, cpu_cached=False)
    order = sorted((e for e in range(n) if load[e]), key=lambda e: (-load[e], e))
    assert [e for e in sorted(order, key=lambda e: p.start[e])] == order
    assert p.makespan == pytest.approx(sum(cost.gpu(load[e]) for e in order))
    # nothing cached, no transfers: the CPU runs them back to back, lowest load first
    p = so.simulate(load, [False] * n, cost, transfers=False)
    assert p.makespan == pytest.approx(sum(cost.cpu(l) for l in load if l))
    assert sorted((e for e in range(n) if load[e]), key=lambda e: p.start[e]) == sorted(
        (e for e in range(n) if load[e]), key=lambda e: (load[e], e))
    # one uncached expert: min(CPU time, transfer + GPU time)
    for l in (1, 4, 40):
        p, which = so.hybrid_schedule([l], [False], cost)
        assert p.makespan == pytest.approx(min(cost.cpu(l), cost.transfer + cost.gpu(l)))
    # not activated experts stay untouched
    p, _ = so.hybrid_schedule(load, [True, False] * 3 + [True], cost)
    assert p.device[1] == -1 and p.device[5] == -1 and p.start[1] == -1 and p.transfer_start[5] == -1


def check_valid(load, cached, cost, plan):
    n = len(load)
    active = [e for e in range(n) if load[e] > 0]
    assert all(plan.device[e] == -1 for e in range(n) if e not in active)
    assert all(plan.device[e] in (GPU0, GPU1, CPU) for e in active)          # every activated expert once
    for e in active:
        dur = cost.cpu(load[e]) if plan.device[e] == CPU else cost.gpu(load[e])
        assert plan.end[e] == pytest.approx(plan.start[e] + dur) and plan.start[e] >= 0
        if plan.device[e] == GPU0:
            assert cached[e] and plan.transfer_start[e] == -1
        if plan.device[e] == GPU1:                                              # not before its weights are there
            assert not cached[e] and plan.start[e] >= plan.transfer_start[e] + cost.transfer - 1e-12
        if plan.device[e] == CPU:
            assert plan.transfer_start[e] == -1
    for dev in ((GPU0, GPU1), (CPU,)):                                         # a timeline does one thing at a time
        iv = sorted((plan.start[e], plan.end[e]) for e in active if plan.device[e] in dev)
        assert all(a[1] <= b[0] + 1e-12 for a, b in zip(iv, iv[1:]))
    tr = sorted(plan.transfer_start[e] for e in active if plan.transfer_start[e] >= 0)
    assert all(b - a >= cost.transfer - 1e-12 for a, b in zip(tr, tr[1:]))
    assert plan.makespan == pytest.approx(max([0.0] + [plan.end[e] for e in active]))


def lower_bound(load, cached, cost):
    """min over all device assignments of a bound no schedule with that assignment can beat"""
    active = [e for e in range(len(load)) if load[e] > 0]
    best = np.inf
    for on_cpu in itertools.product([False, True], repeat=len(active)):
        cpu_t = sum(cost.cpu(load[e]) for e, c in zip(active, on_cpu) if c)
        gpu = [e for e, c in zip(active, on_cpu) if not c]
        gpu_t = sum(cost.gpu(load[e]) for e in gpu)
        loaded = [e for e in gpu if not cached[e]]
        if loaded:    # the last transfer ends no earlier than len(loaded) * transfer, then that expert is computed
            gpu_t = max(gpu_t, len(loaded) * cost.transfer + min(cost.gpu(load[e]) for e in loaded))
        best = min(best, max(cpu_t, gpu_t))
    return best


def test_random_instances_valid_bounded_below_and_above():
    rng = np.random.default_rng(0)
    for trial in range(300):
        n = int(rng.integers(1, 8))
        load = rng.integers(0, 9, n).tolist()
        cached = (rng.random(n) < 0.5).tolist()
        cost = so.SchedCost(*(float(v) for v in rng.choice([0.0, 0.5, 1.0, 2.0, 5.0], 5)))
        for flags in so.STRATEGIES:
            check_valid(load, cached, cost, so.simulate(load, cached, cost, **flags))
        plan, which = so.hybrid_schedule(load, cached, cost)
        check_valid(load, cached, cost, plan)
        assert plan.makespan >= lower_bound(load, cached, cost) - 1e-9
        assert plan.makespan <= so.fixed_mapping_makespan(load, cached, cost, True) + 1e-9
        assert plan.makespan <= so.fixed_mapping_makespan(load, cached, cost, False) + 1e-9
