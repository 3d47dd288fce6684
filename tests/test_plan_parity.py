"""The library's planner (C ABI of include/hyp_plan.h) against the Python oracle: the
same partition vectors, nodes and completion times, bit for bit, on seeded random
instances at the paper's sizes and beyond, plus argument checking.  Host code: no GPU."""
import math
import pathlib
import re

import numpy as np
import pytest

import paper_2511_14450_amd as hyp
from paper_2511_14450_amd import binding
from oracle import hyperion_plan as op

ROOT = pathlib.Path(__file__).resolve().parents[1]


def test_library_exports_every_symbol_of_the_plan_header():
    header = (ROOT / "include" / "hyp_plan.h").read_text()
    declared = re.findall(r"HYP_API\s+[\w\s\*]+?\b(\w+)\s*\(", header)
    assert set(declared) == set(binding.EXPORTS_PLAN)
    lib = hyp.load_library()
    for name in declared:
        assert hasattr(lib, name), name


def _instance(rng, N, T, memory):
    f = rng.uniform(0.2, 3.0, N).tolist()
    m = rng.uniform(0.5, 2.0, N).tolist()
    C = rng.uniform(1.0, 5.0, T).tolist()
    if memory == "none":
        M = [math.inf] * T
    elif memory == "tight":
        M = (rng.uniform(0.9, 1.6, T) * sum(m) / T).tolist()
    else:
        M = (rng.uniform(0.3, 0.9, T) * sum(m) / T).tolist()  # mostly infeasible
    return f, m, C, M


@pytest.mark.parametrize("seed", range(60))
def test_hypsplit_equals_oracle_bit_for_bit(seed):
    rng = np.random.default_rng(3000 + seed)
    N = int(rng.integers(1, 81))          # the paper's models have 32 and 40 blocks
    T = int(rng.integers(1, min(N, 6) + 1))
    f, m, C, M = _instance(rng, N, T, ("none", "tight", "short")[seed % 3])
    eps = float(10.0 ** rng.integers(-9, -1))
    want_p, want_tau = op.hypsplit_dp(f, m, C, M, eps)
    got_p, got_tau = hyp.hypsplit_dp(f, m, C, M, eps)
    assert got_p == want_p
    assert got_tau == want_tau  # same binary-search sequence, same doubles


@pytest.mark.parametrize("seed", range(40))
def test_hypsplit_against_the_plain_min_max_definition(seed):
    """The library's planner against the optimisation problem itself, with no dynamic programme in
    between: every partition vector of a small instance is tried (Sec. IV-A's objective and memory
    constraint), and the library must return a feasible vector whose largest tier load is that
    minimum, with tau* at most eps above it."""
    rng = np.random.default_rng(5000 + seed)
    N = int(rng.integers(2, 12))
    T = int(rng.integers(1, min(N, 4) + 1))
    f, m, C, M = _instance(rng, N, T, ("none", "tight", "short")[seed % 3])
    eps = 1e-9
    p_best, load_best = op.best_partition_by_enumeration(f, m, C, M)
    p, tau = hyp.hypsplit_dp(f, m, C, M, eps)
    if p_best is None:
        assert p is None
        return
    assert p is not None
    b = [0] + p + [N]
    assert all(b[j] < b[j + 1] for j in range(T))
    assert all(sum(m[b[j]:b[j + 1]]) <= M[j] for j in range(T))
    assert max(op.tier_loads(p, f, C)) == pytest.approx(load_best, rel=1e-12)
    assert -1e-12 <= tau - load_best <= eps + 1e-12


def test_hypsplit_zero_cost_blocks_and_ties():
    # zero-cost blocks make many cuts equally good: the kept one must be the oracle's
    f = [0.0, 2.0, 0.0, 0.0, 2.0, 0.0, 2.0, 0.0]
    m = [1.0] * 8
    for C in ([1.0, 1.0, 1.0], [2.0, 1.0, 2.0]):
        for M in ([8.0] * 3, [3.0, 3.0, 3.0]):
            assert hyp.hypsplit_dp(f, m, C, M, 1e-6) == op.hypsplit_dp(f, m, C, M, 1e-6)


def test_hypsplit_paper_sized_example():
    # 40 blocks, three tiers with Table I's TOPS and memory: 6 / 15 / 19 blocks without
    # memory pressure; 8 GB on tier 1 holding at most 5 blocks of 1.4 GB moves the cut
    f = [1.0] * 40
    assert hyp.hypsplit_dp(f, [0.0] * 40, [67.0, 157.0, 200.0], [8.0, 16.0, 32.0], 1e-9)[0] == [6, 21]
    p, tau = hyp.hypsplit_dp(f, [1.4] * 40, [67.0, 157.0, 200.0], [8.0, 16.0, 32.0], 1e-9)
    assert p == op.hypsplit_dp(f, [1.4] * 40, [67.0, 157.0, 200.0], [8.0, 16.0, 32.0], 1e-9)[0]
    assert p is None  # 5 + 11 + 22 = 38 blocks at most: the model does not fit, as the oracle says too


@pytest.mark.parametrize("bad", [
    dict(f=[1.0, -1.0]), dict(f=[1.0, math.nan]), dict(m=[1.0, -0.5]), dict(C=[0.0, 1.0]),
    dict(C=[1.0, math.inf]), dict(M=[1.0, math.nan]), dict(eps=0.0), dict(eps=-1.0),
])
def test_hypsplit_rejects_bad_arguments(bad):
    args = dict(f=[1.0, 2.0], m=[1.0, 1.0], C=[1.0, 2.0], M=[4.0, 4.0], eps=1e-3)
    args.update(bad)
    with pytest.raises(hyp.HypError) as e:
        hyp.hypsplit_dp(args["f"], args["m"], args["C"], args["M"], args["eps"])
    assert e.value.status == binding.HYP_EINVAL


def test_hypsplit_more_tiers_than_blocks_is_rejected():
    with pytest.raises(hyp.HypError):
        hyp.hypsplit_dp([1.0], [1.0], [1.0, 1.0], [1.0, 1.0], 1e-3)


@pytest.mark.parametrize("seed", range(40))
def test_hypsched_equals_oracle(seed):
    rng = np.random.default_rng(4000 + seed)
    K = int(rng.integers(0, 9))
    C = rng.choice([1.0, 2.0, 4.0], K).tolist()
    M_avail = rng.uniform(0, 4, K).tolist()
    available = (rng.uniform(size=K) < 0.8).tolist()
    F_run = rng.choice([0.0, 1.0, 2.0], K).tolist()
    F_wait = rng.choice([0.0, 2.0, 4.0], K).tolist()
    assert hyp.hypsched_rt(2.0, 1.5, C, M_avail, available, F_run, F_wait) == \
        op.hypsched_rt(2.0, 1.5, C, M_avail, available, F_run, F_wait)


@pytest.mark.parametrize("seed", range(20))
def test_queue_model_equals_oracle_bit_for_bit(seed):
    rng = np.random.default_rng(5000 + seed)
    T = int(rng.integers(1, 4))
    n = int(rng.integers(1, 120))
    lam = float(rng.choice([0.2, 1.0, 5.0]))               # the paper's 0.2 tasks / s and heavier loads
    arrivals = np.cumsum(rng.exponential(1.0 / lam, n))
    if seed % 4 == 0:
        arrivals = np.round(arrivals)                        # equal arrival times: tie-breaking by task index
    arrivals = arrivals.tolist()
    F = rng.uniform(1.0, 8.0, T).tolist()
    m_act = rng.uniform(0.5, 1.5, T).tolist()
    Cjk = [rng.choice([1.0, 1.5, 2.0, 3.0], int(rng.integers(1, 4))).tolist() for _ in range(T)]
    Mjk = [rng.uniform(1.0, 6.0, len(c)).tolist() for c in Cjk]
    transfer = rng.uniform(0.0, 0.5, T - 1).tolist()
    available = None if seed % 3 else [[bool(x) for x in (rng.uniform(size=len(c)) < 0.85)] for c in Cjk]
    want = op.simulate_tiers(arrivals, F, m_act, Cjk, Mjk, transfer, available)
    got = hyp.hypsched_simulate(arrivals, F, m_act, Cjk, Mjk, transfer, available)
    assert got[0] == want[0]
    assert got[1] == want[1]


def test_queue_model_rejects_bad_arguments():
    with pytest.raises(hyp.HypError):
        hyp.hypsched_simulate([0.0], [1.0], [0.0], [[0.0]], [[1.0]], [])
    with pytest.raises(ValueError):
        hyp.hypsched_simulate([0.0], [1.0, 1.0], [0.0, 0.0], [[1.0], [1.0]], [[1.0], [1.0]], [])
