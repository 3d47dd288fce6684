"""TEST INFRASTRUCTURE - plain, slow Python of the paper's two scheduling algorithms.

Only tests, the smoke check and the CPU-baseline leg of the benchmark may import
this module; the library's own planner (C++) shares no code with it.

    hypsplit_dp      Sec. IV-A, Algorithm 1: binary search on the target latency tau
                     around the dynamic-programming feasibility check P_check(tau)
                     (the DP(j, n) transition and its base case), partition by
                     backtracking the predecessor table.
    hypsched_rt      Sec. IV-B, Algorithm 2: one pass over the nodes of a tier, the
                     available node with the smallest (queued + new) / C wins.
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
    """DP(j, n) and predecessor P(j, n) of the decision problem for target latency tau."""
    N, T = len(f), len(C)
    S_f, S_m = prefix_sums(f), prefix_sums(m)
    DP = [[False] * (N + 1) for _ in range(T + 1)]
    P = [[-1] * (N + 1) for _ in range(T + 1)]
    DP[0][0] = True
    for j in range(1, T + 1):
        for n in range(j, N + 1):
            for k in range(j - 1, n):
                if DP[j - 1][k]:
                    L_j = (S_f[n] - S_f[k]) / C[j - 1]
                    U_j = S_m[n] - S_m[k]
                    if L_j <= tau and U_j <= M[j - 1]:
                        DP[j][n] = True
                        P[j][n] = k
                        break
    return DP, P


def backtrack(P, T: int, N: int) -> List[int]:
    """p_1 .. p_{T-1} from the predecessor table of a feasible check."""
    p = [0] * (T + 1)
    p[T] = N
    n = N
    for j in range(T, 0, -1):
        n = P[j][n]
        p[j - 1] = n
    assert p[0] == 0
    return p[1:T]


def hypsplit_dp(f, m, C, M, eps: float) -> Tuple[Optional[List[int]], float]:
    """Algorithm 1.  Returns (p*, tau*); p* is None if no partition is feasible."""
    N, T = len(f), len(C)
    assert 1 <= T <= N and eps > 0
    S_f = prefix_sums(f)
    tau_low, tau_high = 0.0, S_f[N] / min(C)
    p_star, tau_star = None, tau_high
    DP, P = p_check(tau_high, f, m, C, M)
    if DP[T][N]:
        p_star = backtrack(P, T, N)
    while (tau_high - tau_low) > eps:
        tau_mid = (tau_low + tau_high) / 2
        DP, P = p_check(tau_mid, f, m, C, M)
        if DP[T][N]:
            tau_star = tau_mid
            tau_high = tau_mid
            p_star = backtrack(P, T, N)
        else:
            tau_low = tau_mid
    return p_star, tau_star


def tier_loads(p: Sequence[int], f, C) -> List[float]:
    """L_j(p) for j = 1..T."""
    N, T = len(f), len(C)
    b = [0] + list(p) + [N]
    S_f = prefix_sums(f)
    return [(S_f[b[j + 1]] - S_f[b[j]]) / C[j] for j in range(T)]


def hypsched_rt(F_new: float, m_act: float, C, M_avail, available, F_run_rem, F_wait) -> Optional[int]:
    """Algorithm 2 for one tier.  Per node k: capacity C[k], available memory M_avail[k],
    availability flag, remaining workload of the running task, summed workload of the
    waiting tasks.  Returns the index of k* or None."""
    min_cost, k_star = float("inf"), None
    for k in range(len(C)):
        if available[k] and M_avail[k] >= m_act:
            F_queued = F_run_rem[k] + F_wait[k]
            cost = (F_queued + F_new) / C[k]
            if cost < min_cost:
                min_cost, k_star = cost, k
    return k_star


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
