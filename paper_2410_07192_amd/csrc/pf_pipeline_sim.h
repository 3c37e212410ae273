// Dependency simulation of a 1F1B pipeline with one stage that holds back at its bubble instructions (bubble
// characterisation, Sec. 4.2).  Header-only: the planner runs it on given times, the runtime runs it with the
// probed stage's instructions executed for real on the device.
#pragma once

#include <algorithm>
#include <cstdint>
#include <vector>

namespace pf {

// One iteration of a stage in 1F1B order.  op: 0 forward, 1 backward, 2 bubble; idx: microbatch or window.
struct StageOp { int32_t op, idx; };

inline std::vector<StageOp> stage_ops(int32_t p, int32_t m, int32_t s) {
  std::vector<StageOp> v;
  const int32_t warm = std::min(p - s, m);
  for (int32_t j = 0; j < warm; ++j) v.push_back({0, j});
  int32_t k = 0;
  if (p - s - 1 > 0) v.push_back({2, k++});
  int32_t next_f = warm;
  bool after_fwd = true;
  for (int32_t j = 0; j < m; ++j) {
    if (!after_fwd) v.push_back({2, k++});
    v.push_back({1, j});
    after_fwd = false;
    if (next_f < m) {
      v.push_back({0, next_f++});
      after_fwd = true;
    }
  }
  if (s > 0) v.push_back({2, k++});
  return v;
}

// Steady-state period of the pipeline when stage s holds back, at its bubble k, for waits[k] after its
// previous instruction.  Finish times live in flat arrays [iteration][stage][microbatch]; stages are swept
// round-robin, each running as far as its dependencies allow (the schedule is a DAG, so every sweep advances).
// run_s(op, microbatch, earliest start) -> finish time of that instruction of stage s (a negative value aborts
// and is returned); the other stages take tf / tb.
template <class RunS>
int64_t period_with_waits(int32_t p, int32_t m, int64_t tf, int64_t tb, int32_t s, const std::vector<int64_t>& waits,
                          const std::vector<std::vector<StageOp>>& ops, RunS&& run_s) {
  constexpr int32_t ITER = 4;
  const size_t per_it = (size_t)p * m;
  std::vector<int64_t> fin_f(ITER * per_it, -1), fin_b(ITER * per_it, -1);
  std::vector<int32_t> pc(p, 0), it(p, 0);
  std::vector<int64_t> free_at(p, 0), hold(p, 0);
  int64_t end_it[ITER] = {0, 0, 0, 0};
  int32_t live = p;
  while (live > 0) {
    for (int32_t q = 0; q < p; ++q) {
      while (it[q] < ITER) {
        const StageOp o = ops[q][pc[q]];
        if (o.op == 2) {
          if (q == s) hold[q] = free_at[q] + waits[o.idx];
        } else {
          const size_t at = (size_t)it[q] * per_it + (size_t)q * m + o.idx;
          int64_t dep = 0;
          if (o.op == 0 && q > 0) dep = fin_f[at - m];
          if (o.op == 1 && q < p - 1) dep = fin_b[at + m];
          if (dep < 0) break;   // producer not simulated yet
          const int64_t start = std::max(std::max(free_at[q], hold[q]), dep);
          int64_t end = start + (o.op == 0 ? tf : tb);
          if (q == s) {
            end = run_s(o.op, o.idx, start);
            if (end < 0) return end;
          }
          (o.op == 0 ? fin_f : fin_b)[at] = end;
          free_at[q] = end;
          if (end > end_it[it[q]]) end_it[it[q]] = end;
        }
        if (++pc[q] == (int32_t)ops[q].size()) {
          pc[q] = 0;
          if (++it[q] == ITER) --live;
        }
      }
    }
  }
  return end_it[ITER - 1] - end_it[ITER - 2];
}

inline int64_t period_with_waits(int32_t p, int32_t m, int64_t tf, int64_t tb, int32_t s, const std::vector<int64_t>& waits,
                                 const std::vector<std::vector<StageOp>>& ops) {
  return period_with_waits(p, m, tf, tb, s, waits, ops,
                           [&](int32_t op, int32_t, int64_t start) { return start + (op == 0 ? tf : tb); });
}

}  // namespace pf
