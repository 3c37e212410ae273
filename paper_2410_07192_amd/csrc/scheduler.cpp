// Fill-job Scheduler (Sec. 4.4) and the event-driven simulation of job arrivals and completions (Sec. 5.1).
// Host-only, integer-only.  A policy is a score per (waiting job, device that became free); scores are
// reciprocals of positive integers (or minus the arrival time), so "largest score" is decided by comparing
// the integers: nothing is rounded and every schedule is reproducible bit for bit.
#include "pf_internal.h"

#include <algorithm>
#include <vector>

namespace {

// The integer whose smallest value wins under `policy` for job j offered to device dev.
//   FIFO: the arrival time;  SJF: min over devices of the processing time (score 1 / min(j.proc_times));
//   MAKESPAN: max(proc[j][dev], longest remaining busy time of any device) (score 1 / max(...)).
inline int64_t policy_key(int32_t policy, const pf_job* jobs, const int64_t* proc, int32_t n_dev, int32_t j, int32_t dev,
                          int64_t longest_rem) {
  const int64_t* row = proc + (size_t)j * n_dev;
  if (policy == PF_POLICY_FIFO) return jobs[j].arrival_ns;
  if (policy == PF_POLICY_SJF) return *std::min_element(row, row + n_dev);
  return std::max(row[dev], longest_rem);
}

}  // namespace

extern "C" {

int32_t pf_job_time(const pf_bubble* B, int32_t nB, const pf_node* F, int32_t nF, int64_t samples_per_replica,
                    int64_t total_samples, int64_t iter_ns, int64_t fill_ppm, int64_t switch_ns, int64_t* proc_ns) {
  if (!proc_ns || samples_per_replica <= 0 || total_samples <= 0 || iter_ns <= 0)
    return pf::fail(PF_ERR_ARG, "pf_job_time: bad argument");
  int32_t n_chunks = 0, replicas = 0;
  const int32_t rc = pf_plan_bubbles(B, nB, F, nF, fill_ppm, switch_ns, 0, nullptr, 0, &n_chunks, &replicas);
  if (rc != PF_OK && rc != PF_ERR_CAPACITY) return rc;   // message already set by the planner
  int64_t n_fill = 0;
  for (int32_t i = 0; i < nB; ++i) n_fill += B[i].fillable ? 1 : 0;
  const int64_t cycles = (n_chunks + n_fill - 1) / n_fill;
  const __int128 per_pass = (__int128)replicas * samples_per_replica;
  const __int128 passes = ((__int128)total_samples + per_pass - 1) / per_pass;
  const __int128 t = passes * cycles * iter_ns;
  if (t > (__int128)INT64_MAX) return pf::fail(PF_ERR_ARG, "pf_job_time: result does not fit 64 bits");
  *proc_ns = (int64_t)t;
  return PF_OK;
}

int32_t pf_sched_simulate(int32_t policy, const pf_job* jobs, int32_t n_jobs, int32_t n_dev, const int64_t* proc_ns,
                          pf_job_run* runs, int64_t* makespan_ns, int64_t* sum_completion_ns) {
  if (policy < PF_POLICY_FIFO || policy > PF_POLICY_MAKESPAN || !jobs || n_jobs <= 0 || n_dev <= 0 || !proc_ns || !runs)
    return pf::fail(PF_ERR_ARG, "pf_sched_simulate: bad argument");
  for (int32_t j = 0; j < n_jobs; ++j) {
    if (jobs[j].arrival_ns < 0) return pf::fail(PF_ERR_ARG, "pf_sched_simulate: negative arrival time");
    for (int32_t d = 0; d < n_dev; ++d)
      if (proc_ns[(size_t)j * n_dev + d] <= 0)
        return pf::fail(PF_ERR_ARG, "pf_sched_simulate: processing times must be positive");
  }
  std::vector<int32_t> by_arrival(n_jobs);
  for (int32_t j = 0; j < n_jobs; ++j) by_arrival[j] = j;
  std::stable_sort(by_arrival.begin(), by_arrival.end(),
                   [&](int32_t a, int32_t b) { return jobs[a].arrival_ns < jobs[b].arrival_ns; });
  std::vector<int64_t> free_at(n_dev, 0);
  std::vector<int32_t> waiting;
  int32_t next = 0, placed = 0;
  int64_t now = 0;
  while (placed < n_jobs) {
    // admit what has arrived; if nothing can start now, jump to the next arrival or completion
    auto admit = [&]() {
      while (next < n_jobs && jobs[by_arrival[next]].arrival_ns <= now) waiting.push_back(by_arrival[next++]);
    };
    admit();
    const bool idle_dev = std::any_of(free_at.begin(), free_at.end(), [&](int64_t f) { return f <= now; });
    if (waiting.empty() || !idle_dev) {
      int64_t t = INT64_MAX;
      if (next < n_jobs) t = std::min(t, jobs[by_arrival[next]].arrival_ns);
      for (int64_t f : free_at)
        if (f > now) t = std::min(t, f);
      now = std::max(now, t);
      admit();
    }
    for (int32_t dev = 0; dev < n_dev && !waiting.empty(); ++dev) {
      if (free_at[dev] > now) continue;
      int64_t longest_rem = 0;
      for (int64_t f : free_at) longest_rem = std::max(longest_rem, f - now);
      size_t pick = 0;
      for (size_t w = 1; w < waiting.size(); ++w) {
        const int32_t a = waiting[w], b = waiting[pick];
        const int64_t ka = policy_key(policy, jobs, proc_ns, n_dev, a, dev, longest_rem);
        const int64_t kb = policy_key(policy, jobs, proc_ns, n_dev, b, dev, longest_rem);
        if (ka < kb || (ka == kb && (jobs[a].arrival_ns < jobs[b].arrival_ns ||
                                     (jobs[a].arrival_ns == jobs[b].arrival_ns && a < b))))
          pick = w;
      }
      const int32_t j = waiting[pick];
      waiting.erase(waiting.begin() + (long)pick);
      runs[j].device = dev;
      runs[j].start_ns = now;
      runs[j].finish_ns = now + proc_ns[(size_t)j * n_dev + dev];
      free_at[dev] = runs[j].finish_ns;
      ++placed;
    }
  }
  int64_t mk = 0;
  __int128 sum = 0;
  for (int32_t j = 0; j < n_jobs; ++j) {
    mk = std::max(mk, runs[j].finish_ns);
    sum += runs[j].finish_ns - jobs[j].arrival_ns;
  }
  if (makespan_ns) *makespan_ns = mk;
  if (sum_completion_ns) *sum_completion_ns = (int64_t)sum;
  return PF_OK;
}

}  // extern "C"
