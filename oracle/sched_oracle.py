"""CPU oracle of the hybrid CPU-GPU scheduling simulation (HybriMoE, Section IV-B).

TEST INFRASTRUCTURE ONLY: imported by tests; the library's own planner (hmoe_schedule_simulate) is
written separately and shares nothing with this file.

What the paper fixes (Section IV-B, priority rules and the simulation paragraphs):
  * the activated experts are split into a GPU queue (experts cached on the GPU, by load descending) and a
    CPU queue (uncached experts, by load ascending);
  * three timelines are filled step by step: CPU compute, GPU compute, host-to-GPU transfer; each step takes
    the timeline that becomes free first and gives it its next operation;
  * GPU: the highest-load expert of its queue; CPU: the lowest-load uncached expert and, once no uncached
    expert is left, the lowest-load cached expert of the GPU queue; transfer: the highest-load uncached
    expert, which then enters the GPU queue at its place in descending load order;
  * a transferred expert cannot be computed on the GPU before its transfer has finished;
  * the simulation ends when every activated expert has been computed.
The cost model of the paper's worked example (GPU time constant, CPU time proportional to the load, fixed
transfer time) is the linear model used here: time = base + per_token * load.

Readings where the paper is silent (also listed in the design notes):
  * timelines that are free at the same time act in the order CPU, GPU, transfer (the order in which the
    paper names them); equal loads are ordered by expert id (lower id first in both queues);
  * one transfer at a time; an expert leaves the CPU queue when its transfer STARTS;
  * the GPU takes the highest-load expert of its queue whose weights have arrived; if only experts still in
    flight remain it waits for the first to arrive;
  * the CPU takes over only experts that were cached from the start (never one that was just transferred);
  * "evaluate scheduling strategies": four rule sets are simulated and the one with the smallest makespan is
    the plan (see STRATEGIES); two of them are the fixed mappings the paper compares against, so the plan is
    never worse than either under the same cost model.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence

ON_GPU_CACHED, ON_GPU_LOADED, ON_CPU = 0, 1, 2


@dataclass
class SchedCost:
    gpu_base: float
    gpu_per_token: float
    cpu_base: float
    cpu_per_token: float
    transfer: float

    def gpu(self, load: int) -> float:
        return self.gpu_base + self.gpu_per_token * load

    def cpu(self, load: int) -> float:
        return self.cpu_base + self.cpu_per_token * load


@dataclass
class SchedPlan:
    device: List[int]             # per expert: ON_* or -1 (not activated)
    start: List[float]            # compute start / end per expert (-1 if not activated)
    end: List[float]
    transfer_start: List[float]   # -1 where no transfer
    makespan: float


def simulate(load: Sequence[int], cached: Sequence[bool], cost: SchedCost, cpu_uncached: bool = True,
             cpu_cached: bool = True, transfers: bool = True) -> SchedPlan:
    """One run of the three-timeline simulation.  The switches remove an operation from the rules: the CPU
    computing uncached experts, the CPU taking over cached experts when it has nothing else, transfers."""
    n = len(load)
    active = [e for e in range(n) if load[e] > 0]
    device = [-1] * n
    start = [-1.0] * n
    end = [-1.0] * n
    xfer = [-1.0] * n
    arrive = {e: 0.0 for e in active if cached[e]}          # when an expert's weights are on the GPU
    gpu_q = sorted(arrive, key=lambda e: (-load[e], e))
    cpu_q = sorted((e for e in active if not cached[e]), key=lambda e: (load[e], e))
    t_cpu = t_gpu = t_pcie = 0.0
    left = len(active)
    while left:
        options = []   # (time at which the timeline could act, rank in the tie order, name)
        if (cpu_uncached and cpu_q) or (cpu_cached and not (cpu_uncached and cpu_q) and any(cached[e] for e in gpu_q)):
            options.append((t_cpu, 0, "cpu"))
        if gpu_q:
            options.append((max(t_gpu, min(arrive[e] for e in gpu_q)), 1, "gpu"))
        if transfers and cpu_q:
            options.append((t_pcie, 2, "pcie"))
        if not options:
            raise ValueError("the switched-off operations leave an expert that nothing may compute")
        when, _, who = min(options)
        if who == "cpu":
            if cpu_uncached and cpu_q:
                e = cpu_q.pop(0)                                        # lowest-load uncached expert
            else:
                e = min((x for x in gpu_q if cached[x]), key=lambda x: (load[x], x))   # lowest-load cached one
                gpu_q.remove(e)
            device[e], start[e] = ON_CPU, when
            end[e] = t_cpu = when + cost.cpu(load[e])
            left -= 1
        elif who == "gpu":
            e = min((x for x in gpu_q if arrive[x] <= when), key=lambda x: (-load[x], x))
            gpu_q.remove(e)
            device[e], start[e] = (ON_GPU_CACHED if cached[e] else ON_GPU_LOADED), when
            end[e] = t_gpu = when + cost.gpu(load[e])
            left -= 1
        else:
            e = max(cpu_q, key=lambda x: (load[x], -x))                  # highest-load uncached expert
            cpu_q.remove(e)
            xfer[e] = when
            arrive[e] = t_pcie = when + cost.transfer
            gpu_q.append(e)
            gpu_q.sort(key=lambda x: (-load[x], x))
    return SchedPlan(device, start, end, xfer, max([0.0] + [end[e] for e in active]))


# The paper runs the simulation "to evaluate scheduling strategies" before executing; the strategies tried
# here, in this order (the first with the smallest makespan wins): the full rule set; the same without the
# CPU taking over cached experts; the two fixed mappings of Fig. 2 (uncached experts all on the CPU, no
# transfers; no CPU at all, every uncached expert loaded on demand).
STRATEGIES = (dict(cpu_uncached=True, cpu_cached=True, transfers=True),
              dict(cpu_uncached=True, cpu_cached=False, transfers=True),
              dict(cpu_uncached=True, cpu_cached=False, transfers=False),
              dict(cpu_uncached=False, cpu_cached=False, transfers=True))


def hybrid_schedule(load: Sequence[int], cached: Sequence[bool], cost: SchedCost):
    """Returns (plan, index of the winning strategy)."""
    best, which = None, -1
    for i, flags in enumerate(STRATEGIES):
        plan = simulate(load, cached, cost, **flags)
        if best is None or plan.makespan < best.makespan:
            best, which = plan, i
    return best, which


def fixed_mapping_makespan(load: Sequence[int], cached: Sequence[bool], cost: SchedCost, uncached_on_cpu: bool) -> float:
    """Makespan of the two static mappings the paper compares against (Section II-B / Fig. 2): every uncached
    expert computed on the CPU while the GPU computes the cached ones, or every uncached expert loaded on
    demand (one after the other) and computed on the GPU after the cached ones."""
    active = [e for e in range(len(load)) if load[e] > 0]
    t_gpu = sum(cost.gpu(load[e]) for e in active if cached[e])
    misses = [e for e in active if not cached[e]]
    if uncached_on_cpu:
        return max(t_gpu, sum(cost.cpu(load[e]) for e in misses))
    t_arrive = 0.0
    for e in sorted(misses, key=lambda x: (-load[x], x)):
        t_arrive += cost.transfer
        t_gpu = max(t_gpu, t_arrive) + cost.gpu(load[e])
    return t_gpu
