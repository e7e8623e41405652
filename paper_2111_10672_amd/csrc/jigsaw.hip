// Iteration-level placement of training tasks (Sec. 3 of the paper, "Scheduling Algorithm") and its gang
// baseline.  Host code only; it lives in this library because its inputs are what the library measures (a step's
// time and workspace per depth) and its callers are the same.  The rules are stated with the declaration in
// spb.h; this file is one way to carry them out: a device's busy intervals are kept sorted, so the earliest gap is
// one sweep, and the ready queue is an ordered set.
#include <algorithm>
#include <cmath>
#include <set>
#include <tuple>
#include <utility>
#include <vector>

#include "model.h"

namespace spb {
namespace {

struct Device {
  std::vector<std::pair<double, double>> busy;  // disjoint [start, end), sorted by start (and so by end)

  // first interval that ends after t: everything before it lies wholly before t
  std::vector<std::pair<double, double>>::const_iterator first_after(double t) const {
    return std::upper_bound(busy.begin(), busy.end(), t, [](double v, const std::pair<double, double>& iv) { return v < iv.second; });
  }
  // earliest t >= ready with [t, t + d) free
  double earliest(double ready, double d) const {
    double t = ready;
    for (auto it = first_after(ready); it != busy.end(); ++it) {
      if (it->second <= t) continue;
      if (it->first >= t + d) break;
      t = it->second;
    }
    return t;
  }
  bool free_at(double t, double d) const {
    const auto it = first_after(t);
    return it == busy.end() || it->first >= t + d;
  }
  void take(double start, double end) {
    auto it = std::lower_bound(busy.begin(), busy.end(), std::make_pair(start, end));
    busy.insert(it, {start, end});
  }
};

struct Progress {               // of one job's current iteration
  double release = 0.0;         // earliest start of its tasks
  int pending = 0;              // tasks not placed yet
  double latest_end = 0.0;
};

int validate(const spb_sched_job* jobs, int n_jobs, int n_machines, double gamma, double capacity, bool gang) {
  if (n_machines < 1 || !(gamma >= 0.0) || !(capacity >= 0.0)) { set_error("spb_schedule_tasks: n_machines %d, gamma %g, capacity %g", n_machines, gamma, capacity); return SPB_ERR_INVALID_ARG; }
  for (int j = 0; j < n_jobs; ++j) {
    const spb_sched_job& q = jobs[j];
    if (q.workers < 1 || !q.durations || !q.resources || q.iterations < 0 || !(q.arrival >= 0.0) || !(q.model_size >= 0.0)) {
      set_error("spb_schedule_tasks: job %d: workers %d, iterations %d, arrival %g, model size %g or a null array", j, q.workers, q.iterations, q.arrival, q.model_size);
      return SPB_ERR_INVALID_ARG;
    }
    for (int w = 0; w < q.workers; ++w)
      if (!(q.durations[w] > 0.0) || !std::isfinite(q.durations[w]) || !(q.resources[w] >= 0.0) || !(q.resources[w] <= capacity)) {
        set_error("spb_schedule_tasks: job %d worker %d: duration %g, resource %g (capacity %g)", j, w, q.durations[w], q.resources[w], capacity);
        return SPB_ERR_INVALID_ARG;
      }
    if (gang && q.workers > n_machines) { set_error("spb_schedule_tasks: job %d: a gang of %d workers on %d devices", j, q.workers, n_machines); return SPB_ERR_INVALID_ARG; }
  }
  return SPB_OK;
}

void place_tasks(const spb_sched_job* jobs, int n_jobs, int n_machines, double gamma, std::vector<spb_sched_task>& out) {
  std::vector<Device> dev(n_machines);
  std::vector<Progress> prog(n_jobs);
  std::vector<std::vector<int>> last(n_jobs);                  // device of each worker's previous iteration
  using Key = std::tuple<double, int, int, int>;               // (-resource * duration, job, iteration, worker)
  std::set<Key> ready;
  auto release_iteration = [&](int j, int i, double when) {
    prog[j].release = when; prog[j].pending = jobs[j].workers; prog[j].latest_end = 0.0;
    for (int w = 0; w < jobs[j].workers; ++w) ready.insert(Key(-(jobs[j].resources[w] * jobs[j].durations[w]), j, i, w));
  };
  for (int j = 0; j < n_jobs; ++j) {
    last[j].assign(jobs[j].workers, -1);
    if (jobs[j].iterations > 0) release_iteration(j, 0, jobs[j].arrival);
  }
  while (!ready.empty()) {
    const Key k = *ready.begin();
    ready.erase(ready.begin());
    const int j = std::get<1>(k), i = std::get<2>(k), w = std::get<3>(k);
    const spb_sched_job& q = jobs[j];
    const double d = q.durations[w];
    const int prev = i > 0 ? last[j][w] : -1;
    int best_m = -1; double best_start = 0.0;
    for (int m = 0; m < n_machines; ++m) {
      const double when = prog[j].release + (m == prev ? 0.0 : gamma * q.model_size);
      const double start = dev[m].earliest(when, d);
      // earlier start wins; at the same start the previous device, then the lower index (m ascends)
      if (best_m < 0 || start < best_start || (start == best_start && m == prev)) { best_m = m; best_start = start; }
    }
    spb_sched_task t;
    t.job = j; t.iteration = i; t.worker = w; t.machine = best_m; t.moved = (i > 0 && best_m != prev) ? 1 : 0;
    t.start = best_start; t.end = best_start + d; t.held_until = t.end;
    dev[best_m].take(t.start, t.end);
    out.push_back(t);
    last[j][w] = best_m;
    prog[j].latest_end = prog[j].pending == q.workers ? t.end : std::max(prog[j].latest_end, t.end);
    if (--prog[j].pending == 0 && i + 1 < q.iterations) release_iteration(j, i + 1, prog[j].latest_end);
  }
}

void place_gangs(const spb_sched_job* jobs, int n_jobs, int n_machines, double gamma, std::vector<spb_sched_task>& out) {
  std::vector<Device> dev(n_machines);
  std::vector<std::vector<int>> last(n_jobs);
  std::vector<double> weight(n_jobs), slowest(n_jobs);
  using Key = std::tuple<double, int, int>;                    // (-(sum of resources) * slowest duration, job, iteration)
  std::set<Key> ready;
  std::vector<double> release(n_jobs, 0.0);
  for (int j = 0; j < n_jobs; ++j) {
    const spb_sched_job& q = jobs[j];
    last[j].assign(q.workers, -1);
    double sum = 0.0, mx = 0.0;
    for (int w = 0; w < q.workers; ++w) { sum += q.resources[w]; mx = std::max(mx, q.durations[w]); }
    weight[j] = sum * mx; slowest[j] = mx;
    if (q.iterations > 0) { release[j] = q.arrival; ready.insert(Key(-weight[j], j, 0)); }
  }
  std::vector<double> candidates, earliest_gap;
  std::vector<int> assign, free_list;
  while (!ready.empty()) {
    const Key k = *ready.begin();
    ready.erase(ready.begin());
    const int j = std::get<1>(k), i = std::get<2>(k);
    const spb_sched_job& q = jobs[j];
    const double rel = release[j], moved_ready = rel + gamma * q.model_size, hold = slowest[j];
    candidates.clear();
    candidates.push_back(rel); candidates.push_back(moved_ready);
    for (const Device& dv : dev)
      for (auto it = dv.first_after(rel); it != dv.busy.end(); ++it) candidates.push_back(it->second);
    std::sort(candidates.begin(), candidates.end());
    // Fewer than q.workers devices are free before the time by which that many have had their first gap of this
    // length: earlier candidates cannot succeed and are not tried.
    earliest_gap.clear();
    for (const Device& dv : dev) earliest_gap.push_back(dv.earliest(rel, hold));
    std::nth_element(earliest_gap.begin(), earliest_gap.begin() + (q.workers - 1), earliest_gap.end());
    const double not_before = earliest_gap[q.workers - 1];
    double t_found = 0.0; bool found = false;
    for (double t : candidates) {
      if (t < not_before) continue;
      free_list.clear();
      for (int m = 0; m < n_machines; ++m) if (dev[m].free_at(t, hold)) free_list.push_back(m);
      assign.assign(q.workers, -1);
      int unplaced = q.workers;
      for (int w = 0; w < q.workers; ++w) {              // keep the previous device where it is free at t
        const int prev = i > 0 ? last[j][w] : -1;
        auto it = prev >= 0 ? std::find(free_list.begin(), free_list.end(), prev) : free_list.end();
        if (it != free_list.end()) { assign[w] = prev; free_list.erase(it); --unplaced; }
      }
      if (unplaced > 0 && (t < moved_ready || (int)free_list.size() < unplaced)) continue;
      size_t next = 0;
      for (int w = 0; w < q.workers; ++w) if (assign[w] < 0) assign[w] = free_list[next++];   // the others move
      t_found = t; found = true;
      break;
    }
    if (!found) return;   // cannot happen: at the last candidate every device is free (validate bounds the gang)
    for (int w = 0; w < q.workers; ++w) {
      const int prev = i > 0 ? last[j][w] : -1;
      spb_sched_task t;
      t.job = j; t.iteration = i; t.worker = w; t.machine = assign[w]; t.moved = (i > 0 && assign[w] != prev) ? 1 : 0;
      t.start = t_found; t.end = t_found + q.durations[w]; t.held_until = t_found + hold;
      dev[assign[w]].take(t.start, t.held_until);
      out.push_back(t);
      last[j][w] = assign[w];
    }
    if (i + 1 < q.iterations) { release[j] = t_found + hold; ready.insert(Key(-weight[j], j, i + 1)); }
  }
}

}  // namespace
}  // namespace spb

extern "C" int spb_schedule_tasks(const spb_sched_job* jobs, int32_t n_jobs, int32_t n_machines, double gamma, double capacity,
                                  int32_t gang, spb_sched_task* out, int64_t cap, int64_t* n_out, double* makespan) {
  using namespace spb;
  if (n_jobs < 0 || (n_jobs > 0 && !jobs) || !n_out || !makespan || cap < 0 || (cap > 0 && !out)) { set_error("spb_schedule_tasks: null argument or negative count"); return SPB_ERR_INVALID_ARG; }
  if (int rc = validate(jobs, n_jobs, n_machines, gamma, capacity, gang != 0)) return rc;
  int64_t total = 0;
  for (int j = 0; j < n_jobs; ++j) total += (int64_t)jobs[j].workers * jobs[j].iterations;
  *n_out = total;
  if (total > cap) { set_error("spb_schedule_tasks: %lld tasks, room for %lld", (long long)total, (long long)cap); return SPB_ERR_INVALID_ARG; }
  std::vector<spb_sched_task> placed;
  placed.reserve((size_t)total);
  if (gang) place_gangs(jobs, n_jobs, n_machines, gamma, placed);
  else place_tasks(jobs, n_jobs, n_machines, gamma, placed);
  if ((int64_t)placed.size() != total) { set_error("spb_schedule_tasks: internal error, %zu of %lld tasks placed", placed.size(), (long long)total); return SPB_ERR_STATE; }
  double latest = 0.0;
  for (size_t t = 0; t < placed.size(); ++t) { out[t] = placed[t]; latest = std::max(latest, placed[t].held_until); }
  *makespan = latest;
  return SPB_OK;
}
