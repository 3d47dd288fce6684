"""GPU parity at the stage depths the workloads name (10 and 20 blocks, Eq. 1 / Eq. 6
stacking) against the CPU oracle, whole tensors, at a width the oracle can afford.

The bf16 path rounds where it stores 16-bit values (normalised activations, q, k, v,
attention output, SwiGLU output) and keeps the residual stream in fp32 inside a
stage, so its error against the fp32 oracle grows with depth; these tests hold the
deep stages to the same 2e-2 bound as a single block, on the output and on the
update (output - input) with no allowance for the output's own rounding, and print
the measured error of every phase."""
import numpy as np
import pytest

from oracle import hyp_oracle as orc
from workloads import synth
from tests.helpers import make_gpu_stage, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu
TOL = 2e-2

# G = 4 query heads per KV head, head_dim 128 as in the Phi-3-medium-shaped block; projection
# weights N(0, 0.05^2) give sub-layer updates of the same relative size as N(0, 0.02^2) does at
# hidden 5120 (sigma^2 x fan-in of 1.3 against 2.0)
SHAPE = synth.BlockShape(hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=768, dtype="bf16")


def deep_stage(n_layers, lens, steps, seed, flags=0):
    layers = [synth.layer_weights(SHAPE, l, seed, sigma=0.05) for l in range(n_layers)]
    B, T = len(lens), sum(lens)
    cap = max(lens) + steps
    x = synth.hidden_states(T, SHAPE, seed + 1)
    ost = orc.Stage(SHAPE, layers, B, cap, "f32")
    gst = make_gpu_stage(SHAPE, layers, B, cap, T, flags=flags)
    assert gst.uses_mfma()
    errs = {}
    ref = ost.prefill(x, lens)
    got = to_host(gst.prefill(to_dev(x, "bf16"), lens))
    errs["prefill"] = (rel_err(got, ref), rel_err(got - x, ref - x))
    for l in (0, n_layers // 2, n_layers - 1):
        for b in range(B):
            k, v = gst.export_kv(l, b)
            errs[f"kv block {l} request {b}"] = (rel_err(to_host(k), ost.K[l, b, :lens[b]]),
                                                 rel_err(to_host(v), ost.V[l, b, :lens[b]]))
    for s in range(steps):
        xd = synth.hidden_states(B, SHAPE, seed + 2 + s)
        ref = ost.decode_step(xd)
        got = to_host(gst.decode_step(to_dev(xd, "bf16")))
        errs[f"decode step {s}"] = (rel_err(got, ref), rel_err(got - xd, ref - xd))
    for b in range(B):
        k, v = gst.export_kv(n_layers - 1, b)
        n = lens[b] + steps
        errs[f"kv after decode, last block, request {b}"] = (rel_err(to_host(k), ost.K[n_layers - 1, b, :n]),
                                                             rel_err(to_host(v), ost.V[n_layers - 1, b, :n]))
    gst.destroy()
    return errs


@pytest.mark.parametrize("n_layers", [1, 5, 10, 20])
def test_mfma_stage_depth_against_oracle(n_layers):
    # ragged prompts: one token, a tail of one 32-row block, across a 64-row query tile and
    # across a 256-token GEMM tile; 8 cached decode steps
    errs = deep_stage(n_layers, [1, 45, 130, 300], 8, 8100 + n_layers)
    worst = max(max(e) for e in errs.values())
    print(f"\ndepth {n_layers}: prefill out {errs['prefill'][0]:.3e} update {errs['prefill'][1]:.3e}; "
          f"decode out {max(errs[f'decode step {s}'][0] for s in range(8)):.3e} "
          f"update {max(errs[f'decode step {s}'][1] for s in range(8)):.3e}; worst of all {worst:.3e}")
    for what, e in errs.items():
        assert max(e) <= TOL, f"depth {n_layers}, {what}: {e}"


def test_split_k_scratch_is_clean_across_consecutive_steps():
    """The workgroups that finish a split-K row group read the other slices' partial sums
    with plain loads.  Twelve consecutive decode steps with different inputs and an odd
    batch reuse the same scratch lines from whichever compute die finishes a row group; a
    stale line from an earlier step would show as a mismatch against the oracle or
    against the same steps launched kernel by kernel instead of from the recorded graph."""
    import torch
    from paper_2511_14450_amd import binding
    shape = synth.BlockShape(hidden=5120, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=7680, dtype="bf16")  # QKV, gate/up and down all split along K
    layers = [synth.layer_weights(shape, l, 8200, sigma=0.02) for l in range(2)]
    lens = [3, 40, 7, 9, 10]
    x = synth.hidden_states(sum(lens), shape, 8201)
    ost = orc.Stage(shape, layers, 5, 64, "f32")
    a = make_gpu_stage(shape, layers, 5, 64, 80)
    b = make_gpu_stage(shape, layers, 5, 64, 80, flags=binding.HYP_FLAG_NO_GRAPH)
    ref = ost.prefill(x, lens)
    ya, yb = a.prefill(to_dev(x, "bf16"), lens), b.prefill(to_dev(x, "bf16"), lens)
    assert torch.equal(ya, yb) and rel_err(to_host(ya), ref) <= TOL
    for s in range(12):
        # alternate the scale of the input so that consecutive partial sums differ by orders of magnitude
        xd = synth.hidden_states(5, shape, 8202 + s) * np.float32(8.0 if s % 2 else 0.125)
        xd = synth.round_bf16(xd)
        ref = ost.decode_step(xd)
        da, db = a.decode_step(to_dev(xd, "bf16")), b.decode_step(to_dev(xd, "bf16"))
        assert torch.equal(da, db), s
        e = rel_err(to_host(da), ref)
        assert e <= TOL, (s, e)
    a.destroy(); b.destroy()
