"""TEST INFRASTRUCTURE - plain, slow Python of the paper's two scheduling algorithms.

Only tests, the smoke check and the CPU-baseline leg of the benchmark may import
this module; the library's own planner (C++) shares no code with it.

    hypsplit_dp      Sec. IV-A, Algorithm 1: bisection on the target latency tau around
                     the feasibility check P_check(tau), which is evaluated from its
                     state-transition equation as a reachability relation; the partition
                     follows the kept predecessors back from (T, N).
    best_partition_by_enumeration
                     the min-max problem of Sec. IV-A by plain enumeration of every
                     partition vector (small N): what Algorithm 1 approximates.
    hypsched_rt      Sec. IV-B, Algorithm 2: argmin of the expected completion over the
                     eligible nodes of a tier.
    simulate_tiers   the queueing model the scheduler's inputs come from (Sec. IV-B:
                     one FIFO queue per node, T_wait from the remaining and the
                     waiting workloads), run over a list of arrival times.

Notation follows the paper: blocks 1..N with costs f_i, m_i; tiers 1..T with C_j,
M_j; p = (p_1 .. p_{T-1}), p_0 = 0, p_T = N, tier j runs blocks p_{j-1}+1 .. p_j.

Readings where the paper is silent (each listed in the design notes as well):
  * initial bounds: tau_low = 0, tau_high = S_f(N) / min_j C_j (no partition can load
    a tier more than that);
  * the upper bound itself is checked once before the search, so p* is null exactly
    when no partition satisfies the memory limits (every tau in the loop is < tau_high);
  * of several feasible k the DP keeps the first it meets scanning k upward;
  * ties in Algorithm 2 go to the node met first (strict <); no eligible node -> None;
  * a node's available memory at time t is its capacity minus m_act for every task it
    holds (running or waiting); a task occupies its node from assignment to completion;
  * the paper's F_run,rem(t) is C times the time the running task still needs.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple


def prefix_sums(v: Sequence[float]) -> List[float]:
    """S(n) = sum_{i <= n} v_i for n = 0..N, added left to right."""
    s = [0.0]
    for x in v:
        s.append(s[-1] + float(x))
    return s


def p_check(tau: float, f, m, C, M):
    """The decision problem P_check(tau) of Sec. IV-A, read off its state-transition equation

        DP(j, n)  <=>  exists k, j-1 <= k < n :  DP(j-1, k)  and  L <= tau  and  U <= M_j,
                       L = (S_f(n) - S_f(k)) / C_j,   U = S_m(n) - S_m(k),      DP(0, 0) true

    as a reachability relation: reach[j] maps every n for which DP(j, n) holds to the predecessor
    P(j, n) kept for it, the smallest admissible k.  Returns (DP(T, N), reach)."""
    N, T = len(f), len(C)
    S_f, S_m = prefix_sums(f), prefix_sums(m)
    reach = [{0: None}]
    for j in range(1, T + 1):
        C_j, M_j = C[j - 1], M[j - 1]
        before = sorted(reach[j - 1])
        here = {}
        for n in range(j, N + 1):
            admissible = [k for k in before if k < n and (S_f[n] - S_f[k]) / C_j <= tau and S_m[n] - S_m[k] <= M_j]
            if admissible:
                here[n] = admissible[0]
        reach.append(here)
    return N in reach[T], reach


def backtrack(reach, T: int, N: int) -> List[int]:
    """p_1 .. p_{T-1}: follow the predecessors from (T, N) down to (0, 0)."""
    cuts, n = [], N
    for j in range(T, 0, -1):
        n = reach[j][n]
        cuts.append(n)
    assert cuts[-1] == 0
    return cuts[-2::-1]


def hypsplit_dp(f, m, C, M, eps: float) -> Tuple[Optional[List[int]], float]:
    """Algorithm 1: bisect the target latency tau over [0, S_f(N) / min C_j], keeping the partition of
    the last feasible check.  Returns (p*, tau*); p* is None if no partition is feasible."""
    N, T = len(f), len(C)
    assert 1 <= T <= N and eps > 0
    tau_low, tau_high = 0.0, prefix_sums(f)[N] / min(C)
    ok, reach = p_check(tau_high, f, m, C, M)
    p_star, tau_star = (backtrack(reach, T, N) if ok else None), tau_high
    while tau_high - tau_low > eps:
        tau_mid = (tau_low + tau_high) / 2
        ok, reach = p_check(tau_mid, f, m, C, M)
        if ok:
            p_star, tau_star, tau_high = backtrack(reach, T, N), tau_mid, tau_mid
        else:
            tau_low = tau_mid
    return p_star, tau_star


def best_partition_by_enumeration(f, m, C, M) -> Tuple[Optional[List[int]], float]:
    """The optimisation problem itself (the min-max objective of Sec. IV-A over all partition vectors
    that respect the memory limits), by trying every one of the C(N-1, T-1) vectors: the plain
    definition Algorithm 1 approximates to within eps.  Small N only.  Returns (p, max_j L_j(p))
    of the first best vector in lexicographic order, or (None, inf)."""
    from itertools import combinations
    N, T = len(f), len(C)
    best_p, best = None, float("inf")
    for cuts in combinations(range(1, N), T - 1):
        b = (0,) + cuts + (N,)
        if any(sum(m[b[j]:b[j + 1]]) > M[j] for j in range(T)):
            continue
        worst = max(sum(f[b[j]:b[j + 1]]) / C[j] for j in range(T))
        if worst < best:
            best_p, best = list(cuts), worst
    return best_p, best


def tier_loads(p: Sequence[int], f, C) -> List[float]:
    """L_j(p) for j = 1..T."""
    N, T = len(f), len(C)
    b = [0] + list(p) + [N]
    S_f = prefix_sums(f)
    return [(S_f[b[j + 1]] - S_f[b[j]]) / C[j] for j in range(T)]


def hypsched_rt(F_new: float, m_act: float, C, M_avail, available, F_run_rem, F_wait) -> Optional[int]:
    """Algorithm 2 for one tier: k* = argmin over the eligible nodes of the expected completion
    (F_run_rem,k + F_wait,k + F_new) / C_k  (the k* equation of Sec. IV-B); a node is eligible when it is
    available and has m_act of memory free.  Ties go to the node listed first; no eligible node -> None."""
    eligible = [k for k in range(len(C)) if available[k] and M_avail[k] >= m_act]
    if not eligible:
        return None
    completion = {k: (F_run_rem[k] + F_wait[k] + F_new) / C[k] for k in eligible}
    return min(eligible, key=lambda k: (completion[k], k))


def simulate_tiers(arrivals: Sequence[float], F: Sequence[float], m_act: Sequence[float], C, M,
                   transfer: Sequence[float], available=None):
    """Tasks arriving at tier 1 at the given times flow through tiers 1..T; at every tier
    HypSched-RT picks the node, whose FIFO queue the task joins.

      F[j], m_act[j]   workload and memory a task needs at tier j
      C[j][k], M[j][k] capacity and memory of node k of tier j
      transfer[j]      time from the completion at tier j to the arrival at tier j+1
                       (T - 1 entries)

    Returns (node[task][tier], finish[task][tier]); a task that finds no eligible node is
    dropped there (node -1, finish inf for this and the later tiers).  Events are handled
    in time order, earlier task first at equal times.
    """
    import heapq
    T, n_tasks = len(F), len(arrivals)
    # per node: list of (finish time, workload, memory) of the tasks it holds, FIFO order
    held = [[[] for _ in C[j]] for j in range(T)]
    node = [[-1] * T for _ in range(n_tasks)]
    finish = [[float("inf")] * T for _ in range(n_tasks)]
    events = [(float(arrivals[q]), q, 0) for q in range(n_tasks)]
    heapq.heapify(events)
    while events:
        t, q, j = heapq.heappop(events)
        K = len(C[j])
        F_run_rem, F_wait, M_avail = [0.0] * K, [0.0] * K, [0.0] * K
        for k in range(K):
            held[j][k] = [h for h in held[j][k] if h[0] > t]      # finished tasks leave
            used = 0.0
            for idx, (fin, work, mem) in enumerate(held[j][k]):
                used += mem
                if idx == 0:  # the head of a FIFO queue that never idles is the running task
                    F_run_rem[k] = C[j][k] * (fin - t)
                else:
                    F_wait[k] += work
            M_avail[k] = M[j][k] - used
        avail = [True] * K if available is None else available[j]
        k_star = hypsched_rt(F[j], m_act[j], C[j], M_avail, avail, F_run_rem, F_wait)
        if k_star is None:
            continue
        start = held[j][k_star][-1][0] if held[j][k_star] else t
        fin = start + F[j] / C[j][k_star]
        held[j][k_star].append((fin, F[j], m_act[j]))
        node[q][j], finish[q][j] = k_star, fin
        if j + 1 < T:
            heapq.heappush(events, (fin + transfer[j], q, j + 1))
    return node, finish
