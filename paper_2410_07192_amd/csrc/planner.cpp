// Bubble planner: idle windows of a pipeline stage, Algorithm 1 packing, configuration choice,
// and the node chain of a transformer fill job.  Host-only, integer-only (int64 ns / bytes /
// ppm, 128-bit cross products), so results are reproducible bit for bit.
#include "pf_internal.h"
#include "pf_pipeline_sim.h"

#include <algorithm>
#include <vector>

namespace {

// usable duration of a bubble: floor(dur * ppm / 1e6) - switch, clamped at 0 (Sec. 6.1 knob)
inline int64_t usable_ns(int64_t dur, int64_t ppm, int64_t sw) {
  __int128 e = (__int128)dur * ppm / 1000000;
  e -= sw;
  return e > 0 ? (int64_t)e : 0;
}

struct PlanResult {
  int32_t rc = PF_OK;
  int32_t replicas = 0;
  int64_t n_chunks = 0;     // total chunks the plan has (may exceed what was stored)
  int64_t peak_mem = 0;
  int32_t bad_node = -1;
};

// Algorithm 1 (Sec. 4.3).  The replicated chain is never materialised: node j of it is
// F[j % nF].  Chunks beyond `cap` are counted but not stored.
// first_dur >= 0: the job arrives when the first bubble is partly gone; that visit (only) has this duration.
PlanResult plan_impl(const pf_bubble* B, int32_t nB, const pf_node* F, int32_t nF, int64_t ppm,
                     int64_t sw, int32_t first, pf_chunk* out, int64_t cap, int64_t first_dur = -1) {
  PlanResult r;
  std::vector<int32_t> idx;
  std::vector<int64_t> dur, mem;
  for (int32_t i = 0; i < nB; ++i)
    if (B[i].fillable) {
      idx.push_back(i);
      dur.push_back(usable_ns(B[i].dur_ns, ppm, sw));
      mem.push_back(B[i].free_bytes);
    }
  const int32_t n = (int32_t)idx.size();
  if (n == 0 || first < 0 || first >= n) {
    r.rc = PF_ERR_ARG;
    return r;
  }
  __int128 total = 0, chain = 0;
  for (int64_t d : dur) total += d;
  for (int32_t j = 0; j < nF; ++j) chain += F[j].dur_ns;
  // replication loop of the listing: F' grows while dur(F') + dur(F) < sum(B)
  int64_t k = 1;
  if (chain > 0) {
    while ((__int128)k * chain + chain < total) {
      ++k;
      if (k > (int64_t)1 << 24) { r.rc = PF_ERR_ARG; return r; }
    }
  }
  if (k * (int64_t)nF > (int64_t)0x7fffffff) { r.rc = PF_ERR_ARG; return r; }
  r.replicas = (int32_t)k;
  const int64_t n_nodes = k * nF;

  int64_t pos = 0, slot = first;
  int32_t b = first, empty_run = 0;
  while (pos < n_nodes) {
    const int64_t begin = pos;
    int64_t cd = 0, cm = 0;
    const int64_t limit = (r.n_chunks == 0 && first_dur >= 0) ? usable_ns(first_dur, ppm, sw) : dur[b];
    while (pos < n_nodes) {
      const pf_node& nd = F[pos % nF];
      if (!(cd + nd.dur_ns < limit && nd.mem_bytes <= mem[b])) break;
      cd += nd.dur_ns;
      if (nd.mem_bytes > cm) cm = nd.mem_bytes;
      ++pos;
    }
    if (r.n_chunks < cap && out) {
      pf_chunk& c = out[r.n_chunks];
      c.bubble = idx[b];
      c.cycle = (int32_t)(slot / n);
      c.node_begin = (int32_t)begin;
      c.node_end = (int32_t)pos;
      c.dur_ns = cd;
      c.mem_bytes = cm;
    }
    ++r.n_chunks;
    if (cm > r.peak_mem) r.peak_mem = cm;
    if (pos == begin) {
      // a whole cycle took nothing: this node fits nowhere.  The shortened first visit of a job handed over in the
      // middle of a bubble says nothing about what a whole bubble holds and does not count.
      const bool shortened = first_dur >= 0 && r.n_chunks == 1;
      if (!shortened && ++empty_run >= n) {
        r.rc = PF_ERR_INFEASIBLE;
        r.bad_node = (int32_t)(pos % nF);
        return r;
      }
    } else {
      empty_run = 0;
    }
    b = (b + 1 == n) ? 0 : b + 1;
    ++slot;
  }
  return r;
}

using pf::StageOp;
using pf::stage_ops;
using pf::period_with_waits;

bool bad_bubbles(const pf_bubble* B, int32_t nB) {
  if (!B || nB <= 0) return true;
  for (int32_t i = 0; i < nB; ++i)
    if (B[i].dur_ns < 0 || B[i].free_bytes < 0) return true;
  return false;
}

bool bad_nodes(const pf_node* F, int32_t nF) {
  if (!F || nF <= 0) return true;
  for (int32_t i = 0; i < nF; ++i)
    if (F[i].dur_ns < 0 || F[i].mem_bytes < 0) return true;
  return false;
}

}  // namespace

extern "C" {

int32_t pf_schedule_1f1b(int32_t p, int32_t m, int32_t s, int64_t tf, int64_t tb, int64_t free_bytes,
                         int32_t fill_gaps, int64_t min_window, pf_bubble* out, int32_t cap,
                         int32_t* n_out) {
  if (p < 1 || m < 1 || s < 0 || s >= p || tf < 0 || tb < 0 || free_bytes < 0 || cap < 0 || !n_out ||
      (cap > 0 && !out))
    return pf::fail(PF_ERR_ARG, "pf_schedule_1f1b: bad argument");
  // Times follow from the dependency rules with zero communication: backward j of stage s
  // starts at p*tf + (p-1-s)*tb + j*(tf+tb); stage s issues min(p-s, m) forwards first.
  const int64_t period = tf + tb;
  const int64_t T = (int64_t)(m + p - 1) * period;
  const int32_t warm = (p - s - 1 < m) ? p - s - 1 : m;
  const int64_t b0 = (int64_t)p * tf + (int64_t)(p - 1 - s) * tb;
  int32_t n = 0;
  auto put = [&](int64_t a, int64_t e, int32_t kind) {
    if (e <= a) return;
    if (n < cap) {
      pf_bubble& w = out[n];
      w.start_ns = a;
      w.dur_ns = e - a;
      w.free_bytes = free_bytes;
      w.kind = kind;
      w.fillable = (kind != PF_BUBBLE_GAP) ? 1 : ((fill_gaps && e - a >= min_window) ? 1 : 0);
    }
    ++n;
  };
  const int32_t n_fwd_first = (p - s < m) ? p - s : m;
  put((int64_t)(s + n_fwd_first) * tf, b0, PF_BUBBLE_FWD_BWD);
  // the last `warm` backwards (all but the first when warm == m) have no forward before them
  for (int32_t j = (warm < m ? m - warm : 1); j < m; ++j) {
    const int64_t prev_end = b0 + (int64_t)(j - 1) * period + tb;
    put(prev_end, prev_end + tf, PF_BUBBLE_GAP);
  }
  put(b0 + (int64_t)(m - 1) * period + tb, T + (int64_t)s * tf, PF_BUBBLE_FILL_DRAIN);
  *n_out = n;
  if (n > cap) return pf::fail(PF_ERR_CAPACITY, "pf_schedule_1f1b: %d windows, capacity %d", n, cap);
  return PF_OK;
}

int32_t pf_schedule_gpipe(int32_t p, int32_t m, int32_t s, int64_t tf, int64_t tb, int64_t free_bytes,
                          pf_bubble* out, int32_t cap, int32_t* n_out) {
  if (p < 1 || m < 1 || s < 0 || s >= p || tf < 0 || tb < 0 || free_bytes < 0 || cap < 0 || !n_out ||
      (cap > 0 && !out))
    return pf::fail(PF_ERR_ARG, "pf_schedule_gpipe: bad argument");
  const int64_t period = tf + tb;
  const int64_t T = (int64_t)(m + p - 1) * period;
  int32_t n = 0;
  auto put = [&](int64_t a, int64_t d, int32_t kind) {
    if (d <= 0) return;
    if (n < cap) out[n] = pf_bubble{a, d, free_bytes, kind, 1};
    ++n;
  };
  put((int64_t)(s + m) * tf, (int64_t)(p - s - 1) * period, PF_BUBBLE_FWD_BWD);
  put(T + (int64_t)s * tf - (int64_t)s * period, (int64_t)s * period, PF_BUBBLE_FILL_DRAIN);
  *n_out = n;
  if (n > cap) return pf::fail(PF_ERR_CAPACITY, "pf_schedule_gpipe: %d windows, capacity %d", n, cap);
  return PF_OK;
}

int32_t pf_plan_bubbles(const pf_bubble* B, int32_t nB, const pf_node* F, int32_t nF, int64_t fill_ppm,
                        int64_t switch_ns, int32_t first_bubble, pf_chunk* out, int32_t cap,
                        int32_t* n_out, int32_t* replicas) {
  return pf_plan_bubbles_from(B, nB, F, nF, fill_ppm, switch_ns, first_bubble, -1, out, cap, n_out, replicas);
}

int32_t pf_plan_bubbles_from(const pf_bubble* B, int32_t nB, const pf_node* F, int32_t nF, int64_t fill_ppm,
                             int64_t switch_ns, int32_t first_bubble, int64_t first_dur_ns, pf_chunk* out,
                             int32_t cap, int32_t* n_out, int32_t* replicas) {
  if (bad_bubbles(B, nB) || bad_nodes(F, nF) || fill_ppm < 0 || fill_ppm > 1000000 || switch_ns < 0 ||
      cap < 0 || !n_out || (cap > 0 && !out))
    return pf::fail(PF_ERR_ARG, "pf_plan_bubbles: bad argument");
  PlanResult r = plan_impl(B, nB, F, nF, fill_ppm, switch_ns, first_bubble, out, cap, first_dur_ns);
  if (replicas) *replicas = r.replicas;
  if (r.rc == PF_ERR_ARG) return pf::fail(PF_ERR_ARG, "pf_plan_bubbles: no fillable bubble, first_bubble out of range, or plan too large");
  if (r.rc == PF_ERR_INFEASIBLE) {
    *n_out = r.bad_node;
    return pf::fail(PF_ERR_INFEASIBLE, "pf_plan_bubbles: node %d (dur %lld ns, mem %lld B) fits no bubble",
                    r.bad_node, (long long)F[r.bad_node].dur_ns, (long long)F[r.bad_node].mem_bytes);
  }
  if (r.n_chunks > 0x7fffffff) return pf::fail(PF_ERR_ARG, "pf_plan_bubbles: plan too large");
  *n_out = (int32_t)r.n_chunks;
  if (r.n_chunks > cap)
    return pf::fail(PF_ERR_CAPACITY, "pf_plan_bubbles: %lld chunks, capacity %d", (long long)r.n_chunks, cap);
  return PF_OK;
}

int32_t pf_probe_bubbles(int32_t p, int32_t m, int32_t s, int64_t tf, int64_t tb, int64_t first_wait,
                         int64_t tol_ppm, int64_t* est, int32_t cap, int32_t* n_out) {
  if (p < 1 || m < 1 || s < 0 || s >= p || tf <= 0 || tb <= 0 || first_wait < 1 || tol_ppm < 0 || cap < 0 || !n_out ||
      (cap > 0 && !est) || (int64_t)p * m > (int64_t)1 << 22)
    return pf::fail(PF_ERR_ARG, "pf_probe_bubbles: bad argument");
  std::vector<std::vector<StageOp>> ops;
  for (int32_t q = 0; q < p; ++q) ops.push_back(stage_ops(p, m, q));
  int32_t n = 0;
  for (const StageOp& o : ops[s]) n += (o.op == 2);
  *n_out = n;
  if (n > cap) return pf::fail(PF_ERR_CAPACITY, "pf_probe_bubbles: %d windows, capacity %d", n, cap);
  std::vector<int64_t> waits(n, 0);
  const int64_t base = period_with_waits(p, m, tf, tb, s, waits, ops);
  const int64_t limit = base + (int64_t)((__int128)base * tol_ppm / 1000000);
  // the pipeline slows down at the latest once one wait exceeds a whole iteration plus the tolerance
  for (int32_t k = 0; k < n; ++k) {
    int64_t w = first_wait;
    for (;;) {
      const int64_t keep = waits[k];
      waits[k] = w;
      const bool slowed = period_with_waits(p, m, tf, tb, s, waits, ops) > limit;
      if (slowed || w > ((int64_t)1 << 60)) {
        waits[k] = keep;
        break;
      }
      w *= 2;
    }
  }
  for (int32_t k = 0; k < n; ++k) est[k] = waits[k];
  return PF_OK;
}

int32_t pf_offload_plan(int32_t p, int32_t m, int32_t s, int64_t tf, int64_t sync_ns, int64_t state_bytes,
                        int64_t d2h, int64_t h2d, int64_t* slice_bytes, int64_t* extra_free, int32_t cap,
                        int32_t* n_windows) {
  if (p < 1 || m < 1 || s < 0 || s >= p || tf <= 0 || sync_ns < 0 || state_bytes < 0 || state_bytes >= ((int64_t)1 << 62) || d2h < 0 || h2d < 0 ||
      !slice_bytes || !n_windows || cap < 0 || (cap > 0 && !extra_free))
    return pf::fail(PF_ERR_ARG, "pf_offload_plan: bad argument");
  constexpr int64_t ALIGN = 256, NS = 1000000000;
  auto moved = [&](int64_t rate, int64_t dur) {
    const __int128 b = (__int128)rate * dur / NS;
    const __int128 lim = (__int128)1 << 62;   // above any state_bytes accepted here, so the clamp never shows
    return (int64_t)((b < lim ? b : lim) / ALIGN * ALIGN);
  };
  const int64_t per_fwd = moved(d2h, tf);
  __int128 total = state_bytes / ALIGN * ALIGN;
  if ((__int128)per_fwd * m < total) total = (__int128)per_fwd * m;
  if (moved(h2d, sync_ns) < total) total = moved(h2d, sync_ns);
  int64_t left = (int64_t)total;
  for (int32_t j = 0; j < m; ++j) {
    slice_bytes[j] = left < per_fwd ? left : per_fwd;
    left -= slice_bytes[j];
  }
  const std::vector<StageOp> ops = stage_ops(p, m, s);
  int32_t n = 0;
  for (const StageOp& o : ops) n += (o.op == 2);
  *n_windows = n;
  if (n > cap) return pf::fail(PF_ERR_CAPACITY, "pf_offload_plan: %d windows, capacity %d", n, cap);
  int64_t gone = 0;
  int32_t k = 0;
  for (const StageOp& o : ops) {
    if (o.op == 0) gone += slice_bytes[o.idx];
    else if (o.op == 2) extra_free[k++] = gone;
  }
  if (s > 0) extra_free[n - 1] = 0;   // the fill-drain window follows the optimizer update: the state is back
  return PF_OK;
}

int32_t pf_select_config(const pf_bubble* B, int32_t nB, const pf_node* const* chains, const int32_t* n_nodes,
                         const int64_t* samples, int32_t n_cfg, int64_t fill_ppm, int64_t switch_ns,
                         int32_t first_bubble, int32_t* best, int32_t* replicas_out, int32_t* cycles_out,
                         int32_t* chunks_out) {
  if (bad_bubbles(B, nB) || !chains || !n_nodes || !samples || n_cfg <= 0 || !best || fill_ppm < 0 ||
      fill_ppm > 1000000 || switch_ns < 0)
    return pf::fail(PF_ERR_ARG, "pf_select_config: bad argument");
  int64_t n_fill = 0;
  for (int32_t i = 0; i < nB; ++i) n_fill += B[i].fillable ? 1 : 0;
  if (n_fill == 0 || first_bubble < 0 || first_bubble >= n_fill)
    return pf::fail(PF_ERR_ARG, "pf_select_config: no fillable bubble or first_bubble out of range");
  *best = -1;
  __int128 best_num = 0;
  int64_t best_cyc = 1, best_peak = 0;
  for (int32_t c = 0; c < n_cfg; ++c) {
    if (replicas_out) replicas_out[c] = 0;
    if (cycles_out) cycles_out[c] = 0;
    if (chunks_out) chunks_out[c] = 0;
    if (bad_nodes(chains[c], n_nodes[c]) || samples[c] < 0)
      return pf::fail(PF_ERR_ARG, "pf_select_config: bad chain %d", c);
    PlanResult r = plan_impl(B, nB, chains[c], n_nodes[c], fill_ppm, switch_ns, first_bubble, nullptr, 0);
    if (r.rc == PF_ERR_INFEASIBLE) continue;
    if (r.rc != PF_OK) return pf::fail(r.rc, "pf_select_config: planning chain %d failed", c);
    const int64_t cyc = (r.n_chunks + n_fill - 1) / n_fill;
    if (replicas_out) replicas_out[c] = r.replicas;
    if (cycles_out) cycles_out[c] = (int32_t)cyc;
    if (chunks_out) chunks_out[c] = (int32_t)r.n_chunks;
    const __int128 num = (__int128)samples[c] * r.replicas;
    bool take = false;
    if (*best < 0) {
      take = true;
    } else {
      const __int128 lhs = num * best_cyc, rhs = best_num * cyc;   // num/cyc vs best_num/best_cyc
      take = lhs > rhs || (lhs == rhs && r.peak_mem < best_peak);
    }
    if (take) {
      *best = c;
      best_num = num;
      best_cyc = cyc;
      best_peak = r.peak_mem;
    }
  }
  if (*best < 0) return pf::fail(PF_ERR_INFEASIBLE, "pf_select_config: no configuration is feasible");
  return PF_OK;
}

int32_t pf_select_config_stream(const pf_bubble* B, int32_t nB, const pf_node* const* chains, const int32_t* n_nodes,
                                const int64_t* samples, int32_t n_cfg, int64_t fill_ppm, int64_t switch_ns,
                                int32_t first_bubble, int32_t horizon_cycles, int32_t* best, int32_t* runs_out,
                                int32_t* cycles_out, int32_t* chunks_out) {
  if (bad_bubbles(B, nB) || !chains || !n_nodes || !samples || n_cfg <= 0 || !best || fill_ppm < 0 ||
      fill_ppm > 1000000 || switch_ns < 0 || horizon_cycles < 1)
    return pf::fail(PF_ERR_ARG, "pf_select_config_stream: bad argument");
  // usable time of one cycle, as Algorithm 1 sees it
  __int128 usable = 0;
  for (int32_t i = 0; i < nB; ++i) {
    if (!B[i].fillable) continue;
    const int64_t e = (int64_t)((__int128)B[i].dur_ns * fill_ppm / 1000000) - switch_ns;
    if (e > 0) usable += e;
  }
  std::vector<std::vector<pf_node>> runs((size_t)n_cfg);
  std::vector<const pf_node*> ptrs((size_t)n_cfg);
  std::vector<int32_t> lens((size_t)n_cfg);
  std::vector<int64_t> smp((size_t)n_cfg);
  for (int32_t c = 0; c < n_cfg; ++c) {
    if (bad_nodes(chains[c], n_nodes[c]) || samples[c] < 0)
      return pf::fail(PF_ERR_ARG, "pf_select_config_stream: bad chain %d", c);
    __int128 dur = 0;
    for (int32_t j = 0; j < n_nodes[c]; ++j) dur += chains[c][j].dur_ns;
    __int128 r = 1;
    if (dur > 0) {
      r = (usable * horizon_cycles + dur - 1) / dur;
      if (r < 1) r = 1;
    }
    if (r * n_nodes[c] > ((__int128)1 << 24))
      return pf::fail(PF_ERR_ARG, "pf_select_config_stream: the run of chain %d would have more than 2^24 nodes", c);
    runs[c].reserve((size_t)(r * n_nodes[c]));
    for (int64_t k = 0; k < (int64_t)r; ++k) runs[c].insert(runs[c].end(), chains[c], chains[c] + n_nodes[c]);
    ptrs[c] = runs[c].data();
    lens[c] = (int32_t)runs[c].size();
    smp[c] = samples[c] * (int64_t)r;
    if (runs_out) runs_out[c] = (int32_t)r;
  }
  return pf_select_config(B, nB, ptrs.data(), lens.data(), smp.data(), n_cfg, fill_ppm, switch_ns, first_bubble, best,
                          nullptr, cycles_out, chunks_out);
}

}  // extern "C"
