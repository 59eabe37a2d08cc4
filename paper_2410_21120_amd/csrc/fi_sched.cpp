// Manager-side scheduling on top of the DAG entry points (Section IV, "Manager": how many models
// one DAG may hold given the device memory; long-running sets are cut into batches that each fit,
// every batch becomes a DAG, and the scheduler runs a fixed number of iterations per DAG before
// swapping in the next one, round robin).  Host logic only: every device step goes through
// fi_build_dag / fi_load / fi_run / fi_unload.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "fi_internal.h"

using namespace fi;

namespace {

double now_ms() {
  using clk = std::chrono::steady_clock;
  return std::chrono::duration<double, std::milli>(clk::now().time_since_epoch()).count();
}

struct Group {
  std::vector<int32_t> members;   // indices into the caller's model array, in the caller's order
  fi_dag* dag = nullptr;
  fi_dag_info info{};
  hipEvent_t loaded = nullptr;    // recorded on the copy stream after the group's load
};

}  // namespace

extern "C" {

fi_status fi_partition(const fi_model_spec* models, int32_t n, const fi_build_opts* opts, uint64_t budget_bytes,
                       int32_t* group_of, int32_t* n_groups) {
  if (!models || n < 1 || !opts || !group_of || !n_groups) { set_error("null argument or no models"); return FI_EINVAL; }
  if (!budget_bytes) { set_error("budget_bytes must be positive"); return FI_EINVAL; }
  // First fit in the caller's order: a model joins the current batch while the batch's exact footprint
  // (weight arena + planned activations + workspace of the compiled DAG) stays inside the budget.
  std::vector<fi_model_spec> cur;
  int32_t g = 0;
  for (int32_t m = 0; m < n; ++m) {
    cur.push_back(models[m]);
    fi_dag_info info{};
    fi_status st = fi_footprint(cur.data(), (int32_t)cur.size(), opts, &info);
    if (st != FI_OK && st != FI_EBUDGET) return st;
    if (st == FI_EBUDGET || info.device_bytes > budget_bytes) {
      if (cur.size() == 1) {
        if (st == FI_OK) set_error("model %d alone needs %llu device bytes, budget is %llu", m,
                                   (unsigned long long)info.device_bytes, (unsigned long long)budget_bytes);
        return FI_EBUDGET;
      }
      ++g;                       // close the batch; the model opens the next one
      cur.clear();
      cur.push_back(models[m]);
      st = fi_footprint(cur.data(), 1, opts, &info);
      if (st != FI_OK) return st;
      if (info.device_bytes > budget_bytes) {
        set_error("model %d alone needs %llu device bytes, budget is %llu", m,
                  (unsigned long long)info.device_bytes, (unsigned long long)budget_bytes);
        return FI_EBUDGET;
      }
    }
    group_of[m] = g;
  }
  *n_groups = g + 1;
  return FI_OK;
}

fi_status fi_round_robin(const fi_model_spec* models, int32_t n, const fi_build_opts* opts, const int32_t* group_of,
                         int32_t n_groups, const fi_sched_opts* sched, const void* d_input, int32_t batch,
                         void* const* d_outputs, void* hip_stream, fi_sched_stats* stats) {
  if (!models || n < 1 || !opts || !group_of || n_groups < 1 || !sched || !d_input || !d_outputs) {
    set_error("null argument"); return FI_EINVAL; }
  if (sched->iterations < 1 || sched->rounds < 1) { set_error("iterations and rounds must be >= 1"); return FI_EINVAL; }
  std::vector<Group> groups((size_t)n_groups);
  for (int32_t m = 0; m < n; ++m) {
    if (group_of[m] < 0 || group_of[m] >= n_groups) { set_error("group_of[%d] = %d outside [0, %d)", m, group_of[m], n_groups); return FI_EINVAL; }
    groups[(size_t)group_of[m]].members.push_back(m);
  }
  for (const Group& g : groups)
    if (g.members.empty()) { set_error("a group has no member"); return FI_EINVAL; }

  hipStream_t compute = static_cast<hipStream_t>(hip_stream);
  hipStream_t copy = nullptr;
  const bool overlap = sched->overlap_load != 0 && n_groups > 1;
  fi_status rc = FI_OK;
  auto cleanup = [&]() {
    for (Group& g : groups) {
      if (g.dag) fi_destroy(g.dag);
      if (g.loaded) (void)hipEventDestroy(g.loaded);
    }
    if (copy) (void)hipStreamDestroy(copy);
  };

  // compile every batch once (host only); the pinned images stay with the handles across rounds
  const double t_begin = now_ms();
  for (Group& g : groups) {
    std::vector<fi_model_spec> specs;
    for (int32_t m : g.members) specs.push_back(models[m]);
    rc = fi_build_dag(specs.data(), (int32_t)specs.size(), opts, &g.dag);
    if (rc != FI_OK) { cleanup(); return rc; }
    (void)fi_query(g.dag, &g.info);
    if (hipEventCreateWithFlags(&g.loaded, hipEventDisableTiming) != hipSuccess) { set_error("hipEventCreate failed"); cleanup(); return FI_EHIP; }
  }
  const double t_built = now_ms();
  uint64_t peak = 0;
  for (int32_t k = 0; k < n_groups; ++k) {
    uint64_t need = groups[(size_t)k].info.device_bytes;
    if (overlap) need += groups[(size_t)((k + 1) % n_groups)].info.device_bytes;   // two batches resident while one loads
    peak = need > peak ? need : peak;
  }
  if (opts->max_device_bytes && peak > opts->max_device_bytes) {
    set_error("round robin keeps up to %llu device bytes resident, budget is %llu", (unsigned long long)peak, (unsigned long long)opts->max_device_bytes);
    cleanup();
    return FI_EBUDGET;
  }
  if (overlap && hipStreamCreateWithFlags(&copy, hipStreamNonBlocking) != hipSuccess) { set_error("hipStreamCreate failed"); cleanup(); return FI_EHIP; }

  double wait_ms = 0.0, run_ms = 0.0;
  int32_t n_loads = 0, n_runs = 0;
  auto load = [&](Group& g) -> fi_status {
    const fi_status st = fi_load(g.dag, overlap ? copy : compute);
    if (st != FI_OK) return st;
    ++n_loads;
    (void)hipEventRecord(g.loaded, overlap ? copy : compute);
    return FI_OK;
  };
  const int32_t total_steps = sched->rounds * n_groups;
  rc = load(groups[0]);   // a single batch stays resident for all rounds
  for (int32_t step = 0; rc == FI_OK && step < total_steps; ++step) {
    Group& g = groups[(size_t)(step % n_groups)];
    // with overlap the next batch travels to the device while this one computes
    if (overlap && step + 1 < total_steps) {
      rc = load(groups[(size_t)((step + 1) % n_groups)]);
      if (rc != FI_OK) break;
    }
    double t0 = now_ms();
    if (overlap) (void)hipStreamWaitEvent(compute, g.loaded, 0);
    std::vector<void*> outs;
    for (int32_t m : g.members) outs.push_back(d_outputs[m]);
    for (int32_t it = 0; it < sched->iterations && rc == FI_OK; ++it) {
      rc = fi_run(g.dag, d_input, batch, outs.data(), compute);
      ++n_runs;
    }
    if (rc != FI_OK) break;
    if (hipStreamSynchronize(compute) != hipSuccess) { set_error("hipStreamSynchronize failed"); rc = FI_EHIP; break; }
    run_ms += now_ms() - t0;
    if (n_groups > 1) {
      t0 = now_ms();
      rc = fi_unload(g.dag);          // swap out; also drains the copy stream, whose load was issued before the runs
      if (rc != FI_OK) break;
      if (!overlap && step + 1 < total_steps) rc = load(groups[(size_t)((step + 1) % n_groups)]);
      wait_ms += now_ms() - t0;
    }
  }
  if (rc == FI_OK && n_groups == 1) rc = fi_unload(groups[0].dag);
  const double t_end = now_ms();
  if (stats) {
    std::memset(stats, 0, sizeof(*stats));
    stats->build_ms = t_built - t_begin;
    stats->total_ms = t_end - t_built;
    stats->run_ms = run_ms;
    stats->swap_ms = wait_ms;
    stats->peak_device_bytes = peak;
    stats->n_loads = n_loads;
    stats->n_runs = n_runs;
    stats->n_groups = n_groups;
  }
  cleanup();
  return rc;
}

}  // extern "C"
