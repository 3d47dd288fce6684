"""Pins of the planner oracle (oracle/hyperion_plan.py) to things other than itself:
brute-force enumeration of every partition, closed forms, the Lindley recursion of a
single FIFO server, and invariants of the queueing model.  No GPU."""
import itertools
import math

import numpy as np
import pytest

from oracle import hyperion_plan as op


def brute_force_partition(f, m, C, M):
    """min over all memory-feasible cut vectors of the largest tier load; every tier
    gets at least one block (the DP's k < n)."""
    N, T = len(f), len(C)
    best, best_p = math.inf, None
    for cuts in itertools.combinations(range(1, N), T - 1):
        b = (0,) + cuts + (N,)
        if any(sum(m[b[j]:b[j + 1]]) > M[j] for j in range(T)):
            continue
        load = max(sum(f[b[j]:b[j + 1]]) / C[j] for j in range(T))
        if load < best:
            best, best_p = load, list(cuts)
    return best_p, best


def random_instance(rng, N, T, tight_memory):
    f = rng.uniform(0.5, 3.0, N).tolist()
    m = rng.uniform(0.5, 2.0, N).tolist()
    C = rng.uniform(1.0, 4.0, T).tolist()
    if tight_memory:
        M = (rng.uniform(0.9, 1.6, T) * sum(m) / T).tolist()
    else:
        M = [1e9] * T
    return f, m, C, M


@pytest.mark.parametrize("seed", range(40))
def test_hypsplit_matches_exhaustive_enumeration(seed):
    rng = np.random.default_rng(1000 + seed)
    N = int(rng.integers(2, 11))
    T = int(rng.integers(1, min(N, 4) + 1))
    f, m, C, M = random_instance(rng, N, T, tight_memory=seed % 2 == 1)
    p_opt, tau_opt = brute_force_partition(f, m, C, M)
    eps = 1e-9
    p, tau = op.hypsplit_dp(f, m, C, M, eps)
    if p_opt is None:
        assert p is None
        return
    assert p is not None and len(p) == T - 1
    b = [0] + p + [N]
    assert all(b[j] < b[j + 1] for j in range(T))
    assert all(sum(m[b[j]:b[j + 1]]) <= M[j] + 1e-12 for j in range(T))
    loads = op.tier_loads(p, f, C)
    assert max(loads) <= tau + 1e-12
    assert -1e-12 <= tau - tau_opt <= eps + 1e-12
    # eps is far below the gap between distinct achievable loads here: the optimum itself
    assert max(loads) == pytest.approx(tau_opt, rel=1e-12)


def test_hypsplit_coarse_epsilon_bound():
    rng = np.random.default_rng(7)
    for _ in range(20):
        f, m, C, M = random_instance(rng, 9, 3, tight_memory=False)
        _, tau_opt = brute_force_partition(f, m, C, M)
        for eps in (0.5, 0.05, 1e-3):
            p, tau = op.hypsplit_dp(f, m, C, M, eps)
            assert max(op.tier_loads(p, f, C)) <= tau + 1e-12
            assert 0 <= tau - tau_opt <= eps + 1e-12


def test_feasibility_is_monotone_in_tau():
    rng = np.random.default_rng(11)
    f, m, C, M = random_instance(rng, 10, 3, tight_memory=True)
    _, tau_opt = brute_force_partition(f, m, C, M)
    assert tau_opt < math.inf
    seen_true = False
    for tau in np.linspace(0.0, 2.0 * tau_opt, 200):
        ok, _ = op.p_check(float(tau), f, m, C, M)
        assert ok == (tau >= tau_opt - 1e-12)
        assert not (seen_true and not ok)
        seen_true = seen_true or ok


def test_closed_forms():
    big = [1e9] * 4
    # one tier: nothing to cut, the load is everything over C_1 (the bound itself is feasible)
    p, tau = op.hypsplit_dp([1.0, 2.0, 3.0], [1, 1, 1], [2.0], [1e9], 1e-6)
    assert p == [] and tau == pytest.approx(3.0, abs=1e-6)
    # equal blocks, equal tiers: equal shares
    p, tau = op.hypsplit_dp([1.0] * 12, [1.0] * 12, [1.0] * 4, big, 1e-6)
    assert p == [3, 6, 9] and tau == pytest.approx(3.0, abs=1e-6)
    # speeds 1 : 2 : 3 take 2, 4, 6 of twelve equal blocks, every load 2
    p, tau = op.hypsplit_dp([1.0] * 12, [1.0] * 12, [1.0, 2.0, 3.0], big[:3], 1e-6)
    assert p == [2, 6] and tau == pytest.approx(2.0, abs=1e-6)
    # T = N: one block per tier, the largest f_i / C_i
    p, tau = op.hypsplit_dp([4.0, 1.0, 9.0], [1, 1, 1], [2.0, 1.0, 3.0], big[:3], 1e-6)
    assert p == [1, 2] and tau == pytest.approx(3.0, abs=1e-6)


def test_memory_limits_force_the_cut_and_infeasible_is_null():
    f, m = [1.0] * 6, [1.0] * 6
    # tier 1 holds one block only although it is the fastest
    p, tau = op.hypsplit_dp(f, m, [100.0, 1.0], [1.0, 10.0], 1e-6)
    assert p == [1] and tau == pytest.approx(5.0, abs=1e-6)
    # six blocks do not fit 2 + 3
    p, tau = op.hypsplit_dp(f, m, [1.0, 1.0], [2.0, 3.0], 1e-6)
    assert p is None and tau == pytest.approx(6.0)


def test_table1_tops_with_uniform_blocks():
    # 40 equal blocks on tiers of 67 / 157 / 200 TOPS (Table I), memory left out: by hand
    # 6/67 = 0.0896, 15/157 = 0.0955, 19/200 = 0.0950; moving any block raises the largest.
    # (Table II prints 20 / 13 / 7 for its unpublished f, m and measured capacities.)
    f, m = [1.0] * 40, [0.0] * 40
    p, tau = op.hypsplit_dp(f, m, [67.0, 157.0, 200.0], [1e9] * 3, 1e-9)
    assert p == [6, 21]
    assert tau == pytest.approx(15.0 / 157.0, abs=1e-9)
    assert brute_force_partition(f, m, [67.0, 157.0, 200.0], [1e9] * 3)[0] == [6, 21]


# ------------------------------------------------------------------ Algorithm 2
def scan_reference(F_new, m_act, C, M_avail, available, F_run, F_wait):
    cost = (np.asarray(F_run) + np.asarray(F_wait) + F_new) / np.asarray(C)
    ok = np.asarray(available, dtype=bool) & (np.asarray(M_avail) >= m_act)
    if not ok.any():
        return None
    cost = np.where(ok, cost, np.inf)
    return int(np.argmin(cost))  # first minimum


@pytest.mark.parametrize("seed", range(30))
def test_hypsched_is_the_first_minimum_over_eligible_nodes(seed):
    rng = np.random.default_rng(2000 + seed)
    K = int(rng.integers(1, 9))
    C = rng.choice([1.0, 2.0, 4.0], K).tolist()
    M_avail = rng.uniform(0, 4, K).tolist()
    available = (rng.uniform(size=K) < 0.8).tolist()
    F_run = rng.choice([0.0, 1.0, 2.0], K).tolist()
    F_wait = rng.choice([0.0, 2.0, 4.0], K).tolist()
    got = op.hypsched_rt(2.0, 1.5, C, M_avail, available, F_run, F_wait)
    assert got == scan_reference(2.0, 1.5, C, M_avail, available, F_run, F_wait)


def test_hypsched_special_cases():
    # idle equal nodes: the first; idle unequal: the fastest
    assert op.hypsched_rt(1.0, 0.0, [2.0, 2.0, 2.0], [1, 1, 1], [True] * 3, [0] * 3, [0] * 3) == 0
    assert op.hypsched_rt(1.0, 0.0, [1.0, 4.0, 2.0], [1, 1, 1], [True] * 3, [0] * 3, [0] * 3) == 1
    # a loaded fast node loses to an idle slow one: (6 + 1) / 4 > 1 / 1
    assert op.hypsched_rt(1.0, 0.0, [1.0, 4.0], [1, 1], [True, True], [0, 2.0], [0, 4.0]) == 0
    # memory and availability filters; nobody eligible
    assert op.hypsched_rt(1.0, 2.0, [1.0, 4.0], [3.0, 1.0], [True, True], [0, 0], [0, 0]) == 0
    assert op.hypsched_rt(1.0, 2.0, [1.0, 4.0], [3.0, 3.0], [False, True], [0, 0], [0, 0]) == 1
    assert op.hypsched_rt(1.0, 2.0, [1.0, 4.0], [1.0, 1.0], [True, True], [0, 0], [0, 0]) is None
    assert op.hypsched_rt(1.0, 0.0, [], [], [], [], []) is None


# ------------------------------------------------------------------ queueing model
def test_single_server_follows_the_lindley_recursion():
    rng = np.random.default_rng(5)
    arrivals = np.cumsum(rng.exponential(1.0 / 0.2, 50)).tolist()  # Poisson, 0.2 tasks / s
    F, C = 12.0, 3.0                                                 # 4 s of service: utilisation 0.8
    node, finish = op.simulate_tiers(arrivals, [F], [0.0], [[C]], [[1.0]], [])
    prev = 0.0
    for a, n, fin in zip(arrivals, node, finish):
        prev = max(a, prev) + F / C
        assert n == [0] and fin[0] == pytest.approx(prev, rel=1e-12)


def test_two_tiers_hand_off_and_fifo_invariants():
    rng = np.random.default_rng(6)
    arrivals = np.cumsum(rng.exponential(2.0, 60)).tolist()
    F, m_act = [6.0, 9.0], [1.0, 1.0]
    C = [[1.0, 2.0, 2.0], [3.0, 1.5]]
    M = [[8.0, 8.0, 8.0], [8.0, 8.0]]
    transfer = [0.25]
    node, finish = op.simulate_tiers(arrivals, F, m_act, C, M, transfer)
    for j in range(2):
        for k in range(len(C[j])):
            mine = sorted((finish[q][j] - F[j] / C[j][k], finish[q][j], q) for q in range(60) if node[q][j] == k)
            for (s0, f0, q0), (s1, f1, q1) in zip(mine, mine[1:]):
                assert s1 >= f0 - 1e-12          # one task at a time per node
    for q in range(60):
        k0, k1 = node[q]
        assert k0 >= 0 and k1 >= 0
        assert finish[q][0] >= arrivals[q] + F[0] / C[0][k0] - 1e-12
        assert finish[q][1] >= finish[q][0] + transfer[0] + F[1] / C[1][k1] - 1e-12
    assert len({n[0] for n in node}) > 1  # the load does spread over nodes


def test_sparse_arrivals_always_take_the_fastest_idle_node():
    arrivals = [100.0 * i for i in range(5)]
    node, finish = op.simulate_tiers(arrivals, [4.0], [0.0], [[1.0, 2.0, 2.0]], [[1.0] * 3], [])
    assert [n[0] for n in node] == [1] * 5
    assert [f[0] for f in finish] == [a + 2.0 for a in arrivals]


def test_memory_holds_tasks_off_a_full_node():
    # three tasks at once, each needs the whole memory of a node: two nodes take one each, the third is dropped
    node, finish = op.simulate_tiers([0.0, 0.0, 0.0], [2.0], [1.0], [[1.0, 1.0]], [[1.0, 1.0]], [])
    assert [n[0] for n in node] == [0, 1, -1]
    assert finish[2][0] == math.inf
    # after the first completes its memory is free again
    node, _ = op.simulate_tiers([0.0, 0.0, 2.5], [2.0], [1.0], [[1.0, 1.0]], [[1.0, 1.0]], [])
    assert [n[0] for n in node] == [0, 1, 0]
