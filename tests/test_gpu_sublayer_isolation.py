"""Localising checks of the MFMA path against the oracle: the block's sub-layers are fused into a
few kernels, so they are isolated through the weights instead of through entry points of their
own - with some projections zeroed a stage exercises only the residual path, only the attention
sub-layer (RMS Norm, QKV, RoPE, cache, attention, O projection) or only the feed-forward sub-layer
(RMS Norm, gate/up, SwiGLU, down projection), on ragged prompts and odd batch widths.  A failure
here names the sub-layer; the exported cache separates the QKV + RoPE part from the attention."""
import numpy as np
import pytest

from oracle import hyp_oracle as orc
from workloads import synth
from tests.helpers import make_gpu_stage, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu
TOL = 2e-2
SHAPE = synth.BlockShape(hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=768, dtype="bf16")
LENS = [1, 45, 130, 300, 64]
STEPS = 3


def run(layers, seed):
    B, T, cap = len(LENS), sum(LENS), max(LENS) + STEPS
    x = synth.hidden_states(T, SHAPE, seed)
    ost = orc.Stage(SHAPE, layers, B, cap, "f32")
    gst = make_gpu_stage(SHAPE, layers, B, cap, T)
    assert gst.uses_mfma()
    outs = [(x, to_host(gst.prefill(to_dev(x, "bf16"), LENS)), ost.prefill(x, LENS))]
    for s in range(STEPS):
        xd = synth.hidden_states(B, SHAPE, seed + 1 + s)
        outs.append((xd, to_host(gst.decode_step(to_dev(xd, "bf16"))), ost.decode_step(xd)))
    return ost, gst, outs


def zeroed(w, names):
    return {k: (np.zeros_like(v) if k in names else v) for k, v in w.items()}


def test_residual_path_alone_is_exact():
    # every projection zero: each sub-layer adds nothing and the stage must hand its input through bit for bit
    layers = [zeroed(synth.layer_weights(SHAPE, l, 8600, sigma=0.05), {"wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"})
              for l in range(2)]
    _, gst, outs = run(layers, 8601)
    for x, got, ref in outs:
        assert np.array_equal(got, x) and np.array_equal(ref, x)
    gst.destroy()


def test_attention_sublayer_alone():
    # w_down = 0: out = x + Wo attention(...); the cache isolates RMS Norm + QKV + RoPE from the attention itself
    layers = [zeroed(synth.layer_weights(SHAPE, l, 8610, sigma=0.05), {"w_down"}) for l in range(2)]
    ost, gst, outs = run(layers, 8611)
    for l in range(2):
        for b in range(len(LENS)):
            k, v = gst.export_kv(l, b)
            n = LENS[b] + STEPS
            assert rel_err(to_host(k), ost.K[l, b, :n]) <= TOL, ("keys after RoPE", l, b)
            assert rel_err(to_host(v), ost.V[l, b, :n]) <= TOL, ("values", l, b)
    for i, (x, got, ref) in enumerate(outs):
        assert rel_err(got - x, ref - x) <= TOL, ("attention update", i)
    gst.destroy()


def test_feed_forward_sublayer_alone():
    # wo = 0: out = x + Wd (silu(Wg r) * (Wu r)), r = RMS Norm of x: no attention result reaches the output
    layers = [zeroed(synth.layer_weights(SHAPE, l, 8620, sigma=0.05), {"wo"}) for l in range(2)]
    _, gst, outs = run(layers, 8621)
    for i, (x, got, ref) in enumerate(outs):
        assert rel_err(got - x, ref - x) <= TOL, ("feed-forward update", i)
    gst.destroy()
