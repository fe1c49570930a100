// Exact solver for the single-layer recomputation policy (Sec. 4.2 of the
// paper: objective (objective2), constraints (cons11)-(cons17), the last-stage
// variant of "Optimizations").  Host code only.
//
// The paper hands the program to an LP/MILP solver.  A layer has n = 13
// operators, so the search is done directly: every retain set S with S_n = 1
// that fits the memory of Eq. (cons16) is visited; for each, the operators that
// have to be regenerated (those backward reads and, transitively, their
// discarded inputs) are given a phase by depth-first search in operator order.
// Eq. (cons12) makes phases non-decreasing along every dependency edge, which
// keeps the tree small; a branch is cut as soon as a communication window
// (cons13), the forward-window memory (cons17) or the best critical-path time
// found so far is exceeded.  Among policies with the same critical-path time the
// one that regenerates the least time in total wins, then the one with the lower
// peak memory, then the one met first (retain sets in increasing mask order,
// earlier phases first).
#include <math.h>
#include <string.h>

#include "../../include/lynx.h"

namespace {

constexpr int kMaxOps = 24;
constexpr double kEps = 1e-12;

struct Search {
  const lynx_policy_problem* p;
  int n;
  uint32_t retain;          // bit i-1: S_i
  uint32_t must;            // bit i-1: OP_i has to be regenerated
  int order[kMaxOps];       // the operators of `must`, ascending
  int count;
  int phase[kMaxOps + 1];   // phase of OP_i while searching (0: none)
  double used[6];           // time placed into each phase
  double fwd_bytes;         // bytes regenerated in phases 1, 2 (per layer)
  double fwd_room;          // what Eq. (cons15) leaves for them (per layer)
  double best;              // best critical-path time so far (over all retain sets)
  double best_total;        // its total regenerated time, and
  double best_peak;         // its peak bytes (tie-breakers)
  bool found;
  lynx_policy out;
};

double peak_of(const Search& s) {
  double kept = 0.0;
  for (int i = 1; i <= s.n; ++i)
    if ((s.retain >> (i - 1)) & 1u) kept += s.p->bytes[i - 1];
  return s.p->m_static + static_cast<double>(s.p->n_layer) * s.p->n_batch * kept +
         (s.p->last_stage ? 0.0 : static_cast<double>(s.p->n_layer) * s.fwd_bytes);
}

void record(Search& s, double critical, double total, double peak) {
  s.best = critical;
  s.best_total = total;
  s.best_peak = peak;
  s.found = true;
  lynx_policy& o = s.out;
  memset(&o, 0, sizeof(o));
  o.retain_mask = (s.retain << 1) | 1u;  // bit 0: the layer input, always the caller's
  for (int k = 0; k < s.count; ++k) {
    const int i = s.order[k];
    o.phase_mask[s.phase[i] - 1] |= 1u << i;
  }
  o.critical_cost = critical;
  o.recompute_cost = total;
  o.peak_bytes = peak;
}

void place(Search& s, int k) {
  if (s.found && s.used[5] > s.best + kEps) return;  // already worse on the critical path
  if (k == s.count) {
    double total = 0.0;
    for (int t = 1; t <= 5; ++t) total += s.used[t];
    const double peak = peak_of(s);
    bool better = !s.found || s.used[5] < s.best - kEps;
    if (!better && fabs(s.used[5] - s.best) <= kEps) {
      if (total < s.best_total - kEps) better = true;
      else if (fabs(total - s.best_total) <= kEps && peak < s.best_peak - 1e-6) better = true;
    }
    if (better) record(s, s.used[5], total, peak);
    return;
  }
  const lynx_policy_problem& p = *s.p;
  const int i = s.order[k];
  // Eq. (cons12): not before any regenerated input
  int first = 1;
  const uint32_t par = p.parents[i - 1];
  for (int j = 1; j < i; ++j)
    if (((par >> j) & 1u) && !((s.retain >> (j - 1)) & 1u) && s.phase[j] > first) first = s.phase[j];
  if (p.last_stage && first < 3) first = 3;
  if ((p.comm_mask >> i) & 1u) first = 5;  // Eq. (cons14)
  const double c = p.cost[i - 1];
  for (int t = first; t <= 5; ++t) {
    if (t <= 4 && s.used[t] + c > p.ctime[t - 1] + kEps) continue;            // Eq. (cons13)
    if (t == 5 && s.found && s.used[5] + c > s.best + kEps) continue;           // cannot tie or improve
    if (t <= 2 && s.fwd_bytes + p.bytes[i - 1] > s.fwd_room + 1e-9) continue;   // Eq. (cons17) in (cons15)
    s.phase[i] = t;
    s.used[t] += c;
    if (t <= 2) s.fwd_bytes += p.bytes[i - 1];
    place(s, k + 1);
    if (t <= 2) s.fwd_bytes -= p.bytes[i - 1];
    s.used[t] -= c;
    s.phase[i] = 0;
  }
}

}  // namespace

extern "C" lynx_status lynx_policy_solve(const lynx_policy_problem* p, lynx_policy* out) {
  if (p == nullptr || out == nullptr || p->cost == nullptr || p->bytes == nullptr || p->parents == nullptr)
    return LYNX_ERR_INVALID_ARG;
  const int n = p->n_ops;
  if (n < 1 || n > kMaxOps || p->n_layer < 1 || p->n_batch < 1) return LYNX_ERR_INVALID_ARG;
  for (int i = 1; i <= n; ++i) {
    if (!(p->cost[i - 1] >= 0.0) || !(p->bytes[i - 1] >= 0.0)) return LYNX_ERR_INVALID_ARG;
    if (p->parents[i - 1] >> i) return LYNX_ERR_INVALID_ARG;  // an input must be an earlier operator (or bit 0)
  }
  for (int t = 0; t < 4; ++t)
    if (!(p->ctime[t] >= 0.0)) return LYNX_ERR_INVALID_ARG;

  Search s;
  memset(&s, 0, sizeof(s));
  s.p = p;
  s.n = n;
  s.best = INFINITY;
  const uint32_t all = n == 32 ? 0xFFFFFFFFu : ((1u << n) - 1u);
  const uint32_t needed = (p->needed_mask >> 1) & all;  // bit i-1: OP_i
  const uint32_t last = 1u << (n - 1);
  const double scale = static_cast<double>(p->n_layer) * p->n_batch;
  for (uint32_t retain = last; retain <= all; ++retain) {
    if (!(retain & last)) continue;  // S_n = 1
    double kept = 0.0;
    for (int i = 1; i <= n; ++i)
      if ((retain >> (i - 1)) & 1u) kept += p->bytes[i - 1];
    const double room = p->m_budget - p->m_static - scale * kept;  // Eq. (cons15), (cons16)
    if (room < -1e-9) continue;
    // what has to come back: needed and discarded, then their discarded inputs
    uint32_t must = needed & ~retain;
    for (int i = n; i >= 1; --i)
      if ((must >> (i - 1)) & 1u) must |= (p->parents[i - 1] >> 1) & ~retain & all;
    s.retain = retain;
    s.must = must;
    s.count = 0;
    for (int i = 1; i <= n; ++i)
      if ((must >> (i - 1)) & 1u) s.order[s.count++] = i;
    s.fwd_bytes = 0.0;
    s.fwd_room = p->last_stage ? 0.0 : room / static_cast<double>(p->n_layer);
    for (int t = 0; t < 6; ++t) s.used[t] = 0.0;
    place(s, 0);
  }
  if (!s.found) return LYNX_ERR_OOM;  // not even the checkpoint fits the budget
  *out = s.out;
  return LYNX_OK;
}

// ---- recomputation-aware model partitioning (Sec. 5) ------------------------------
// The section's greedy search: start from equal shares, evaluate every stage with the
// single-layer policy solver, move one layer from the slowest stage to the fastest,
// keep the move if it is valid and the slowest stage got faster, stop otherwise.
namespace {

struct StageEval {
  bool valid;
  double time;
  lynx_policy policy;
};

StageEval eval_stage(const lynx_partition_problem& pp, int stage, int n_layers) {
  StageEval e;
  memset(&e, 0, sizeof(e));
  e.valid = true;
  if (n_layers == 0) return e;
  lynx_policy_problem p = *pp.layer;
  p.n_layer = n_layers;
  p.n_batch = pp.n_stages - stage;  // forward passes held before the first backward (1F1B)
  p.last_stage = stage == pp.n_stages - 1;
  p.m_static = pp.static_per_layer * n_layers;
  p.m_budget = pp.m_budget;
  if (lynx_policy_solve(&p, &e.policy) != LYNX_OK) {
    e.valid = false;
    return e;
  }
  e.time = n_layers * (pp.t_fwd + pp.t_bwd + e.policy.critical_cost);
  return e;
}

}  // namespace

extern "C" lynx_status lynx_partition_solve(const lynx_partition_problem* pp, int32_t* layers_out,
                                            double* time_out, lynx_policy* policies_out) {
  if (pp == nullptr || pp->layer == nullptr || layers_out == nullptr || time_out == nullptr)
    return LYNX_ERR_INVALID_ARG;
  const int P = pp->n_stages, L = pp->n_total_layers;
  if (P < 1 || P > 64 || L < P || !(pp->t_fwd >= 0.0) || !(pp->t_bwd >= 0.0) || !(pp->static_per_layer >= 0.0))
    return LYNX_ERR_INVALID_ARG;
  {  // argument errors of the layer problem surface here, not as "does not fit"
    lynx_policy_problem probe = *pp->layer;
    probe.n_layer = 1;
    probe.n_batch = 1;
    probe.m_budget = INFINITY;
    lynx_policy ignore;
    const lynx_status st = lynx_policy_solve(&probe, &ignore);
    if (st != LYNX_OK) return st;
  }
  int layers[64], trial[64];
  StageEval cur[64], nxt[64];
  for (int s = 0; s < P; ++s) layers[s] = L / P + (s < L % P ? 1 : 0);  // step (1)
  for (int s = 0; s < P; ++s) {                                         // steps (2), (3)
    cur[s] = eval_stage(*pp, s, layers[s]);
    if (!cur[s].valid) return LYNX_ERR_OOM;
  }
  for (;;) {
    int slow = 0, fast = 0;
    for (int s = 1; s < P; ++s) {
      if (cur[s].time > cur[slow].time) slow = s;
      if (cur[s].time < cur[fast].time) fast = s;
    }
    if (slow == fast || layers[slow] <= 1) break;
    for (int s = 0; s < P; ++s) { trial[s] = layers[s]; nxt[s] = cur[s]; }  // step (4)
    trial[slow] -= 1;
    trial[fast] += 1;
    nxt[slow] = eval_stage(*pp, slow, trial[slow]);
    nxt[fast] = eval_stage(*pp, fast, trial[fast]);
    if (!nxt[slow].valid || !nxt[fast].valid) break;
    double worst = 0.0;
    for (int s = 0; s < P; ++s) worst = nxt[s].time > worst ? nxt[s].time : worst;
    if (worst >= cur[slow].time - kEps) break;
    for (int s = 0; s < P; ++s) { layers[s] = trial[s]; cur[s] = nxt[s]; }
  }
  for (int s = 0; s < P; ++s) {                                         // step (5)
    layers_out[s] = layers[s];
    time_out[s] = cur[s].time;
    if (policies_out != nullptr) policies_out[s] = cur[s].policy;
  }
  return LYNX_OK;
}
