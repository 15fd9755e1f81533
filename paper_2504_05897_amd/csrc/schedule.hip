// Host-side planner: the hybrid CPU-GPU scheduling simulation of Section IV-B.
//
// The paper orders the experts of a layer on three resources with three priority rules -- GPU: experts
// whose weights are on the GPU, highest load first; CPU: experts that are not cached, lowest load first,
// then (with nothing else to do) cached experts, lowest load first; host-to-GPU transfer: uncached
// experts, highest load first, each joining the GPU's list when it has arrived -- and finds the
// allocation by simulating the three timelines: whichever resource is free first gets its next
// operation, until every activated expert has been computed.  Several rule sets are simulated and the
// one that finishes first is the plan.
//
// Nothing here touches the device: the planner works on the per-expert loads that hmoe_permute can copy
// to pinned host memory and on a linear cost model (time = base + per_token * load; one fixed transfer
// time per expert), which is the model of the paper's worked example.  Where the paper is silent:
// resources free at the same time act in the order CPU, GPU, transfer; equal loads go by expert id; one
// transfer at a time, and an expert is out of the CPU's reach once its transfer has started; the GPU
// never idles while an expert whose weights have arrived is waiting; the CPU takes over only experts
// that were cached from the start.
#include <algorithm>

#include "common.h"

namespace hmoe {
namespace {

enum ExpertState { NOT_ACTIVE, WAITING_ON_HOST, ON_GPU, DONE };

struct Simulation {
  int n;
  const int32_t* load;
  const int32_t* cached;
  const hmoe_sched_cost* cost;
  int32_t rules;
  ExpertState state[HMOE_MAX_EXPERTS];
  double arrival[HMOE_MAX_EXPERTS];  // ON_GPU: when the weights are (or will be) there
  int32_t* device;
  double *start, *end, *transfer_start;

  double gpu_time(int e) const { return cost->gpu_base + cost->gpu_per_token * load[e]; }
  double cpu_time(int e) const { return cost->cpu_base + cost->cpu_per_token * load[e]; }

  // the expert of a given state with the lowest / highest load (ties: lower id); -1 if none.
  // only_cached: restrict to experts cached from the start; ready_by: restrict to weights arrived by then.
  int pick(ExpertState s, bool highest, bool only_cached, double ready_by) const {
    int best = -1;
    for (int e = 0; e < n; ++e) {
      if (state[e] != s || (only_cached && !cached[e])) continue;
      if (s == ON_GPU && arrival[e] > ready_by) continue;
      if (best < 0 || (highest ? load[e] > load[best] : load[e] < load[best])) best = e;
    }
    return best;
  }

  // Returns the makespan, or a negative value if the rules leave an expert nothing may compute.
  double run() {
    int left = 0;
    for (int e = 0; e < n; ++e) {
      device[e] = -1;
      start[e] = end[e] = transfer_start[e] = -1.0;
      arrival[e] = 0.0;
      state[e] = load[e] <= 0 ? NOT_ACTIVE : (cached[e] ? ON_GPU : WAITING_ON_HOST);
      left += load[e] > 0;
    }
    const double never = 1e300;
    double cpu_free = 0.0, gpu_free = 0.0, link_free = 0.0, makespan = 0.0;
    while (left > 0) {
      const int host_low = pick(WAITING_ON_HOST, false, false, never);
      const int host_high = pick(WAITING_ON_HOST, true, false, never);
      // what each resource would do next, and when
      int cpu_job = -1;
      if ((rules & HMOE_SCHED_CPU_UNCACHED) && host_low >= 0) cpu_job = host_low;
      else if (rules & HMOE_SCHED_CPU_CACHED) cpu_job = pick(ON_GPU, false, true, never);
      double gpu_at = never;
      for (int e = 0; e < n; ++e)
        if (state[e] == ON_GPU) gpu_at = std::min(gpu_at, arrival[e]);
      const bool gpu_can = gpu_at < never;
      gpu_at = std::max(gpu_at, gpu_free);
      const bool link_can = (rules & HMOE_SCHED_TRANSFERS) && host_high >= 0;

      // earliest first; CPU before GPU before transfer on equal times
      int who = -1;  // 0 CPU, 1 GPU, 2 transfer
      double when = never;
      if (cpu_job >= 0) { who = 0; when = cpu_free; }
      if (gpu_can && gpu_at < when) { who = 1; when = gpu_at; }
      if (link_can && link_free < when) { who = 2; when = link_free; }
      if (who < 0) return -1.0;

      if (who == 0) {
        const int e = cpu_job;
        device[e] = HMOE_ON_CPU;
        start[e] = when;
        end[e] = cpu_free = when + cpu_time(e);
        makespan = std::max(makespan, end[e]);
        state[e] = DONE;
        --left;
      } else if (who == 1) {
        const int e = pick(ON_GPU, true, false, when);
        device[e] = cached[e] ? HMOE_ON_GPU_CACHED : HMOE_ON_GPU_LOADED;
        start[e] = when;
        end[e] = gpu_free = when + gpu_time(e);
        makespan = std::max(makespan, end[e]);
        state[e] = DONE;
        --left;
      } else {
        const int e = host_high;
        transfer_start[e] = when;
        arrival[e] = link_free = when + cost->transfer;
        state[e] = ON_GPU;
      }
    }
    return makespan;
  }
};

int check_args(int32_t n, const int32_t* load, const int32_t* cached, const hmoe_sched_cost* cost, const int32_t* device,
               const double* start, const double* end, const double* transfer_start, const double* makespan) {
  if (n < 0 || n > HMOE_MAX_EXPERTS || !cost || !makespan) return HMOE_ERR_INVALID_ARG;
  if (n > 0 && (!load || !cached || !device || !start || !end || !transfer_start)) return HMOE_ERR_INVALID_ARG;
  const double c[5] = {cost->gpu_base, cost->gpu_per_token, cost->cpu_base, cost->cpu_per_token, cost->transfer};
  for (double v : c)
    if (!(v >= 0.0) || v > 1e100) return HMOE_ERR_INVALID_ARG;
  for (int e = 0; e < n; ++e)
    if (load[e] < 0) return HMOE_ERR_INVALID_ARG;
  return HMOE_OK;
}

}  // namespace
}  // namespace hmoe

extern "C" int32_t hmoe_schedule_simulate(int32_t n_experts, const int32_t* h_load, const int32_t* h_cached,
                                          const hmoe_sched_cost* cost, int32_t rules, int32_t* h_device,
                                          double* h_start, double* h_end, double* h_transfer_start, double* makespan) {
  using namespace hmoe;
  const int rc = check_args(n_experts, h_load, h_cached, cost, h_device, h_start, h_end, h_transfer_start, makespan);
  if (rc != HMOE_OK) return rc;
  if (rules & ~HMOE_SCHED_ALL) return HMOE_ERR_INVALID_ARG;
  Simulation sim{n_experts, h_load, h_cached, cost, rules, {}, {}, h_device, h_start, h_end, h_transfer_start};
  const double t = sim.run();
  if (t < 0.0) return HMOE_ERR_UNSUPPORTED;
  *makespan = t;
  return HMOE_OK;
}

extern "C" int32_t hmoe_schedule_plan(int32_t n_experts, const int32_t* h_load, const int32_t* h_cached,
                                      const hmoe_sched_cost* cost, int32_t* h_device, double* h_start, double* h_end,
                                      double* h_transfer_start, double* makespan, int32_t* rules_out) {
  using namespace hmoe;
  const int rc = check_args(n_experts, h_load, h_cached, cost, h_device, h_start, h_end, h_transfer_start, makespan);
  if (rc != HMOE_OK) return rc;
  // the rule sets tried, in this order; the first with the smallest makespan is the plan.  The last two are
  // the fixed mappings of Fig. 2: uncached experts on the CPU without transfers, and no CPU at all.
  const int32_t candidates[4] = {HMOE_SCHED_ALL, HMOE_SCHED_CPU_UNCACHED | HMOE_SCHED_TRANSFERS, HMOE_SCHED_CPU_UNCACHED,
                                 HMOE_SCHED_TRANSFERS};
  int32_t dev[HMOE_MAX_EXPERTS];
  double st[HMOE_MAX_EXPERTS], en[HMOE_MAX_EXPERTS], tr[HMOE_MAX_EXPERTS];
  double best = -1.0;
  for (int32_t rules : candidates) {
    Simulation sim{n_experts, h_load, h_cached, cost, rules, {}, {}, dev, st, en, tr};
    const double t = sim.run();
    if (t < 0.0) continue;
    if (best < 0.0 || t < best) {
      best = t;
      std::copy(dev, dev + n_experts, h_device);
      std::copy(st, st + n_experts, h_start);
      std::copy(en, en + n_experts, h_end);
      std::copy(tr, tr + n_experts, h_transfer_start);
      if (rules_out) *rules_out = rules;
    }
  }
  if (best < 0.0) return HMOE_ERR_UNSUPPORTED;
  *makespan = best;
  return HMOE_OK;
}
