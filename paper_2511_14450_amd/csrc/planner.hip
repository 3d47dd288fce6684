// Host-side planner: offline partitioning (Sec. IV-A, Algorithm 1), online node
// selection (Sec. IV-B, Algorithm 2) and the per-node FIFO queue model between them.
// No device code; it lives in the stage library so that one shared object serves a node.
#include <cmath>
#include <cstdint>
#include <deque>
#include <limits>
#include <queue>
#include <vector>

#include "hyp_plan.h"

namespace {

// Feasibility check P_check(tau) in O(T N) instead of the transition's O(T N^2):
// with f, m >= 0 the prefix sums are monotone, so for tier j the predicate
//   [(S_f[n] - S_f[k]) / C_j <= tau] and [S_m[n] - S_m[k] <= M_j]
// is monotone in k (false .. false true .. true) and its threshold moves right with n.
// The smallest feasible predecessor of (j, n) is then the first k >= threshold with
// DP(j-1, k) true, found through a "next true at or after" table.  The comparisons are
// the transition's own floating-point expressions, so the decisions - and the
// predecessor kept, the smallest - are those of the plain triple loop.
struct Check {
  int N, T;
  const double *C, *M;
  std::vector<double> Sf, Sm;
  std::vector<int> pred;       // [T+1][N+1]
  std::vector<char> dp;        // [T+1][N+1]
  std::vector<int> next_true;  // [N+2]

  bool ok(int j, int n, int k, double tau) const {
    return (Sf[n] - Sf[k]) / C[j - 1] <= tau && Sm[n] - Sm[k] <= M[j - 1];
  }
  bool run(double tau) {
    const int W = N + 1;
    std::fill(dp.begin(), dp.end(), 0);
    dp[0] = 1;  // DP(0, 0)
    for (int j = 1; j <= T; ++j) {
      const char *prev = &dp[(size_t)(j - 1) * W];
      next_true[N + 1] = N + 1;
      for (int k = N; k >= 0; --k) next_true[k] = prev[k] ? k : next_true[k + 1];
      int thr = j - 1;
      for (int n = j; n <= N; ++n) {
        while (thr < n && !ok(j, n, thr, tau)) ++thr;
        if (thr >= n) continue;  // even the single block n does not fit (thr == n)
        int k = next_true[thr];
        if (k < n) {
          dp[(size_t)j * W + n] = 1;
          pred[(size_t)j * W + n] = k;
        }
      }
    }
    return dp[(size_t)T * W + N] != 0;
  }
  void backtrack(int32_t *p_out) const {
    const int W = N + 1;
    int n = N;
    for (int j = T; j >= 1; --j) {
      n = pred[(size_t)j * W + n];
      if (j >= 2) p_out[j - 2] = n;
    }
  }
};

bool finite_nonneg(double v) { return std::isfinite(v) && v >= 0.0; }

struct Held { double finish, work, mem; };
struct Event {
  double t;
  int task, tier;
  bool operator>(const Event &o) const {
    if (t != o.t) return t > o.t;
    if (task != o.task) return task > o.task;
    return tier > o.tier;
  }
};

int select_node(int K, const double *C, const double *M_avail, const uint8_t *available, const double *F_run,
                const double *F_wait, double F_new, double m_act) {
  double min_cost = std::numeric_limits<double>::infinity();
  int k_star = -1;
  for (int k = 0; k < K; ++k) {
    if ((available && !available[k]) || !(M_avail[k] >= m_act)) continue;
    double cost = (F_run[k] + F_wait[k] + F_new) / C[k];
    if (cost < min_cost) { min_cost = cost; k_star = k; }
  }
  return k_star;
}

}  // namespace

extern "C" {

hyp_status_t hypsplit_dp(int32_t n_blocks, int32_t n_tiers, const double *f, const double *m, const double *C,
                         const double *M, double eps, int32_t *p_out, double *tau_out, int32_t *feasible_out) {
  if (!f || !m || !C || !M || !tau_out || !feasible_out) return HYP_EINVAL;
  if (n_tiers < 1 || n_blocks < n_tiers || !(eps > 0.0)) return HYP_EINVAL;
  if (n_tiers > 1 && !p_out) return HYP_EINVAL;
  for (int i = 0; i < n_blocks; ++i)
    if (!finite_nonneg(f[i]) || !finite_nonneg(m[i])) return HYP_EINVAL;
  double c_min = std::numeric_limits<double>::infinity();
  for (int j = 0; j < n_tiers; ++j) {
    if (!std::isfinite(C[j]) || !(C[j] > 0.0) || std::isnan(M[j])) return HYP_EINVAL;
    c_min = std::min(c_min, C[j]);
  }
  Check ck;
  ck.N = n_blocks; ck.T = n_tiers; ck.C = C; ck.M = M;
  try {
    ck.Sf.assign(n_blocks + 1, 0.0); ck.Sm.assign(n_blocks + 1, 0.0);
    ck.pred.assign((size_t)(n_tiers + 1) * (n_blocks + 1), -1);
    ck.dp.assign((size_t)(n_tiers + 1) * (n_blocks + 1), 0);
    ck.next_true.assign(n_blocks + 2, 0);
  } catch (...) { return HYP_ENOMEM; }
  for (int i = 0; i < n_blocks; ++i) {
    ck.Sf[i + 1] = ck.Sf[i] + f[i];
    ck.Sm[i + 1] = ck.Sm[i] + m[i];
  }
  double lo = 0.0, hi = ck.Sf[n_blocks] / c_min, tau_star = hi;
  int found = 0;
  if (ck.run(hi)) { found = 1; if (n_tiers > 1) ck.backtrack(p_out); }
  while (hi - lo > eps) {
    double mid = (lo + hi) / 2;
    if (ck.run(mid)) {
      tau_star = mid; hi = mid; found = 1;
      if (n_tiers > 1) ck.backtrack(p_out);
    } else {
      lo = mid;
    }
  }
  *tau_out = tau_star;
  *feasible_out = found;
  return HYP_OK;
}

hyp_status_t hypsched_rt(int32_t n_nodes, const double *C, const double *M_avail, const uint8_t *available,
                         const double *F_run_rem, const double *F_wait, double F_new, double m_act, int32_t *k_out) {
  if (!k_out || n_nodes < 0) return HYP_EINVAL;
  if (n_nodes > 0 && (!C || !M_avail || !available || !F_run_rem || !F_wait)) return HYP_EINVAL;
  *k_out = select_node(n_nodes, C, M_avail, available, F_run_rem, F_wait, F_new, m_act);
  return HYP_OK;
}

hyp_status_t hypsched_simulate(int32_t n_tasks, const double *arrivals, int32_t n_tiers, const double *F,
                               const double *m_act, const int32_t *nodes_per_tier, const double *C, const double *M,
                               const uint8_t *available, const double *transfer, int32_t *node_out, double *finish_out) {
  if (!arrivals || !F || !m_act || !nodes_per_tier || !C || !M || !node_out || !finish_out) return HYP_EINVAL;
  if (n_tasks < 1 || n_tiers < 1 || (n_tiers > 1 && !transfer)) return HYP_EINVAL;
  try {
    std::vector<int> first(n_tiers + 1, 0);
    for (int j = 0; j < n_tiers; ++j) {
      if (nodes_per_tier[j] < 1) return HYP_EINVAL;
      first[j + 1] = first[j] + nodes_per_tier[j];
    }
    for (int k = 0; k < first[n_tiers]; ++k)
      if (!(C[k] > 0.0)) return HYP_EINVAL;
    std::vector<std::deque<Held>> held(first[n_tiers]);
    std::priority_queue<Event, std::vector<Event>, std::greater<Event>> events;
    for (int q = 0; q < n_tasks; ++q) {
      events.push({arrivals[q], q, 0});
      for (int j = 0; j < n_tiers; ++j) {
        node_out[(size_t)q * n_tiers + j] = -1;
        finish_out[(size_t)q * n_tiers + j] = std::numeric_limits<double>::infinity();
      }
    }
    std::vector<double> F_run, F_wait, M_avail;
    while (!events.empty()) {
      Event e = events.top();
      events.pop();
      const int j = e.tier, K = nodes_per_tier[j], base = first[j];
      F_run.assign(K, 0.0); F_wait.assign(K, 0.0); M_avail.assign(K, 0.0);
      for (int k = 0; k < K; ++k) {
        std::deque<Held> &h = held[base + k];
        // tasks leave when they finish; with FIFO service finish times increase along the queue
        while (!h.empty() && !(h.front().finish > e.t)) h.pop_front();
        double used = 0.0;
        for (size_t i = 0; i < h.size(); ++i) {
          used += h[i].mem;
          if (i == 0) F_run[k] = C[base + k] * (h[i].finish - e.t);  // the head is the running task
          else F_wait[k] += h[i].work;
        }
        M_avail[k] = M[base + k] - used;
      }
      int k_star = select_node(K, C + base, M_avail.data(), available ? available + base : nullptr, F_run.data(),
                               F_wait.data(), F[j], m_act[j]);
      if (k_star < 0) continue;
      std::deque<Held> &h = held[base + k_star];
      double start = h.empty() ? e.t : h.back().finish;
      double fin = start + F[j] / C[base + k_star];
      h.push_back({fin, F[j], m_act[j]});
      node_out[(size_t)e.task * n_tiers + j] = k_star;
      finish_out[(size_t)e.task * n_tiers + j] = fin;
      if (j + 1 < n_tiers) events.push({fin + transfer[j], e.task, j + 1});
    }
  } catch (...) { return HYP_ENOMEM; }
  return HYP_OK;
}

}  // extern "C"
