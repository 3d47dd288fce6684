"""Whole-model chain (stages over consecutive block ranges, Eq. 6) against the oracle:
the chain's greedy tokens and hidden states must be those of the same blocks run by the
oracle with the activations crossing each boundary in the stage dtype."""
import numpy as np
import pytest

from oracle import hyp_oracle as orc
from workloads import synth
from tests.helpers import rel_err, to_dev, to_host
from tests.test_gpu_mfma_parity import SHAPE_G4
from tests.test_gpu_stage_parity import TOL

pytestmark = pytest.mark.gpu


def _chains(shape, n_layers, bounds, batch, cap, max_prefill, seed, sigma):
    import paper_2511_14450_amd as hyp
    layers = [synth.layer_weights(shape, l, seed, sigma=sigma) for l in range(n_layers)]
    gchain = hyp.StageChain(shape, bounds, lambda l: {k: to_dev(v, shape.dtype) for k, v in layers[l].items()},
                            batch, cap, max_prefill)
    ostages = [orc.Stage(shape, layers[lo:hi], batch, cap, "f32") for lo, hi in zip(bounds[:-1], bounds[1:])]
    return gchain, ostages


def _oracle_chain(ostages, x, lens, dtype, decode):
    for st in ostages:
        x = st.decode_step(x) if decode else st.prefill(x, lens)
        if dtype == "bf16":
            x = synth.round_bf16(x)  # what the previous tier sends is in the stage dtype
    return x


def test_chain_of_three_stages_greedy_tokens_fp32():
    # 4 tiny fp32 blocks cut 1 + 2 + 1; closed loop: the picked token's embedding is the next input
    shape = synth.TINY
    seed = 4411
    gchain, ostages = _chains(shape, 4, [0, 1, 3, 4], 1, 64 + 24, 64, seed, 0.02)
    assert [(s.l_start, s.l_end) for s in gchain.stages] == [(0, 1), (1, 3), (3, 4)]
    E, Emb = synth.readout_tables(shape, 512, seed)
    x = synth.hidden_states(64, shape, seed + 1)
    o = _oracle_chain(ostages, x, [64], "f32", False)[-1]
    g = to_host(gchain.prefill(to_dev(x, "f32"), [64]))[-1]
    toks_o, toks_g, gaps, errs = [], [], [], []
    for s in range(24):
        lo, lg = E.astype(np.float64) @ o, E.astype(np.float64) @ g
        top = np.sort(lo)[-2:]
        gaps.append((top[1] - top[0]) / np.abs(lo).max())
        errs.append(rel_err(g, o))
        toks_o.append(int(lo.argmax())); toks_g.append(int(lg.argmax()))
        o = _oracle_chain(ostages, Emb[toks_o[-1]][None], None, "f32", True)[0]
        g = to_host(gchain.decode_step(to_dev(Emb[toks_g[-1]][None], "f32")))[0]
    assert min(gaps) > 1e-3
    assert toks_o == toks_g
    assert max(errs) <= TOL["f32"]
    assert gchain.context_len(0) == 64 + 24
    gchain.destroy()


def test_chain_bf16_mfma_stages_ragged_batch():
    # 5 bf16 blocks on the MFMA path cut 2 + 1 + 2, two ragged requests, prefill + decode
    shape = SHAPE_G4
    seed = 4421
    lens = [70, 33]
    gchain, ostages = _chains(shape, 5, [0, 2, 3, 5], 2, 80, sum(lens), seed, 0.05)
    assert all(s.uses_mfma() for s in gchain.stages)
    x = synth.hidden_states(sum(lens), shape, seed + 1)
    ref = _oracle_chain(ostages, x, lens, "bf16", False)
    got = to_host(gchain.prefill(to_dev(x, "bf16"), lens))
    assert rel_err(got, ref) <= TOL["bf16"]
    for s in range(6):
        xd = synth.hidden_states(2, shape, seed + 2 + s)
        ref = _oracle_chain(ostages, xd, None, "bf16", True)
        got = to_host(gchain.decode_step(to_dev(xd, "bf16")))
        assert rel_err(got, ref) <= TOL["bf16"], s
    gchain.destroy()


def test_chain_rejects_bad_boundaries():
    import paper_2511_14450_amd as hyp
    for bad in ([1, 2], [0], [0, 2, 2], [0, 3, 1]):
        with pytest.raises(ValueError):
            hyp.StageChain(synth.TINY, bad, lambda l: {}, 1, 8, 8)
