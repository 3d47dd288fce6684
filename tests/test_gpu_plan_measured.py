"""HypSplit-DP (Sec. IV-A, Algorithm 1) fed with block costs measured on the device: the f_i
(seconds a block spends on a request) and m_i (bytes a block adds to a stage) that
`measure_block_costs` takes from this library go through the library's planner and through
the oracle's Algorithm 1; both must return the same partition and target latency, and the
chain of stages built on the planned boundaries (Eq. 6) must compute what the oracle's
stages over the same block ranges compute."""
import numpy as np
import pytest

from oracle import hyp_oracle as orc
from oracle import hyperion_plan as oplan
from workloads import synth
from tests.helpers import rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu

SPEC = dict(blocks=7, hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=768, vocab=0)
SHAPE = synth.BlockShape(hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=768, dtype="bf16")


def test_measured_costs_planned_and_run():
    import paper_2511_14450_amd as hyp
    from paper_2511_14450_amd import chain
    prompt, generate, eps = 48, 12, 1e-6
    f1, m1 = chain.measure_block_costs(SPEC, prompt, generate)
    assert 1e-5 < f1 < 1.0, f1                     # a few kernels per block and step: microseconds to milliseconds
    assert m1 >= 2 * SHAPE.params_per_layer(), m1  # at least the block's bf16 weights
    # tiers with Table I's relative capacities; the first tier's memory holds only two blocks
    tiers = [(67.0, 2.5 * m1 / 1e9), (157.0, 64.0), (200.0, 64.0)]
    plan = chain.plan_split(SPEC, tiers, prompt, generate, eps)
    f, m = [plan["f_seconds_per_block"]] * 7, [plan["m_bytes_per_block"]] * 7
    C = [c / 200.0 for c, _ in tiers]
    M = [g * 1e9 for _, g in tiers]
    p_ref, tau_ref = oplan.hypsplit_dp(f, m, C, M, eps)
    assert plan["p"] == p_ref and plan["tau_seconds"] == tau_ref
    assert plan["p"] is not None and sum(plan["blocks_per_tier"]) == 7
    assert plan["blocks_per_tier"][0] <= 2         # the memory limit binds
    loads = [f[0] * n / c for n, c in zip(plan["blocks_per_tier"], C)]
    assert max(loads) <= plan["tau_seconds"] + 1e-12 and plan["tau_seconds"] - max(loads) <= eps + 1e-12

    # the planned chain against the oracle's stages over the same ranges
    bounds = [0] + plan["p"] + [7]
    seed, lens = 8400, [prompt, 17]
    layers = [synth.layer_weights(SHAPE, l, seed, sigma=0.05) for l in range(7)]
    gchain = hyp.StageChain(SHAPE, bounds, lambda l: {k: to_dev(v, "bf16") for k, v in layers[l].items()},
                            2, prompt + generate, sum(lens))
    ostages = [orc.Stage(SHAPE, layers[lo:hi], 2, prompt + generate, "f32") for lo, hi in zip(bounds[:-1], bounds[1:])]

    def oracle_chain(x, decode):
        for st in ostages:
            x = synth.round_bf16(st.decode_step(x) if decode else st.prefill(x, lens))  # a tier hands over bf16
        return x

    x = synth.hidden_states(sum(lens), SHAPE, seed + 1)
    assert rel_err(to_host(gchain.prefill(to_dev(x, "bf16"), lens)), oracle_chain(x, False)) <= 2e-2
    for s in range(4):
        xd = synth.hidden_states(2, SHAPE, seed + 2 + s)
        assert rel_err(to_host(gchain.decode_step(to_dev(xd, "bf16"))), oracle_chain(xd, True)) <= 2e-2, s
    gchain.destroy()
