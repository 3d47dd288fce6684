"""A tier of stage replicas on separate streams driven by HypSched-RT: whichever node
serves a task, its result is the one a lone stage computes, and every choice the tier
made is the oracle's choice for the queue state it saw."""
import numpy as np
import pytest

from oracle import hyp_oracle as orc
from oracle import hyperion_plan as op
from workloads import synth
from tests.helpers import make_gpu_stage, rel_err, to_dev, to_host
from tests.test_gpu_mfma_parity import SHAPE_G2
from tests.test_gpu_stage_parity import TOL

pytestmark = pytest.mark.gpu


def _tier(shape, layers, n_nodes, cap, max_prefill, **kw):
    from paper_2511_14450_amd.tier import Tier
    return Tier(shape, 0, len(layers), lambda l: {k: to_dev(v, shape.dtype) for k, v in layers[l].items()},
                n_nodes, 1, cap, max_prefill, **kw)


@pytest.mark.parametrize("shape,sigma", [(synth.TINY, 0.02), (SHAPE_G2, 0.05)])
def test_any_node_gives_the_lone_stage_result(shape, sigma):
    import torch
    seed, S, steps, n_tasks = 5150, 48, 5, 9
    layers = [synth.layer_weights(shape, l, seed, sigma=sigma) for l in range(2)]
    tier = _tier(shape, layers, 3, S + steps + 1, S)
    xs = [synth.hidden_states(S, shape, seed + 10 + q) for q in range(n_tasks)]
    tasks = [tier.submit(to_dev(x, shape.dtype), [S], steps, work=1.0) for x in xs]
    assert all(t is not None for t in tasks)
    torch.cuda.synchronize()
    assert len({t.node for t in tasks}) >= 2           # equal nodes, queued work: the load spreads
    lone = make_gpu_stage(shape, layers, 1, S + steps + 1, S)
    ost = orc.Stage(shape, layers, 1, S + steps + 1, "f32")
    for q, (x, t) in enumerate(zip(xs, tasks)):
        h = lone.prefill(to_dev(x, shape.dtype), [S])[-1:].contiguous()
        for _ in range(steps):
            h = lone.decode_step(h)
        assert torch.equal(h, t.out), q                 # bit for bit, whichever replica and stream
        if q in (0, n_tasks - 1):                       # and the oracle's value for the same closed loop
            o = ost.prefill(x, [S])[-1:]
            for _ in range(steps):
                o = ost.decode_step(synth.round_bf16(o) if shape.dtype == "bf16" else o)
            assert rel_err(to_host(t.out), o) <= TOL[shape.dtype] * (3 if shape.dtype == "bf16" else 1)
    lone.destroy()
    # every decision against Algorithm 2 as the oracle states it, on the recorded state
    assert len(tier.decisions) == n_tasks
    for d in tier.decisions:
        assert d["k"] == op.hypsched_rt(d["F_new"], d["m_act"], d["C"], d["M_avail"], d["available"],
                                        d["F_run_rem"], d["F_wait"])
    tier.destroy()


def test_capacity_and_availability_steer_the_choice():
    import torch
    shape = synth.TINY
    layers = [synth.layer_weights(shape, 0, 5160)]
    tier = _tier(shape, layers, 3, 40, 32, capacity=[1.0, 4.0, 1.0])
    x = to_dev(synth.hidden_states(32, shape, 5161), "f32")
    # long credited workloads keep the predicted queues busy whatever the GPU has finished
    first = tier.submit(x, [32], 2, work=1000.0)
    assert first.node == 1                               # idle nodes: the fastest
    second = tier.submit(x, [32], 2, work=1000.0)
    assert second.node == 1                              # (1000 + 1000) / 4 < 1000 / 1
    tier.available[1] = False
    third = tier.submit(x, [32], 2, work=1000.0)
    assert third.node == 0                               # fastest is out: first of the equal rest
    tier.available = [False, False, False]
    assert tier.submit(x, [32], 2, work=1.0) is None
    torch.cuda.synchronize()
    for d in tier.decisions:
        assert d["k"] == op.hypsched_rt(d["F_new"], d["m_act"], d["C"], d["M_avail"], d["available"],
                                        d["F_run_rem"], d["F_wait"])
    tier.destroy()
