"""GPU parity of the MFMA path (bf16 stages with head_dim 128) against the CPU
oracle, element by element, on shapes small enough for the oracle yet spanning
several 256-wide tiles, ragged tails and more than one decode chunk."""
import dataclasses

import numpy as np
import pytest

from oracle import hyp_oracle as orc
from workloads import synth
from tests.helpers import make_gpu_stage, rel_err, to_dev, to_host
from tests.test_gpu_stage_parity import check, TOL

pytestmark = pytest.mark.gpu

# G = 2 and G = 4 query heads per KV head; widths are multiples of 256
SHAPE_G2 = synth.BlockShape(hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn_dim=512, dtype="bf16")
SHAPE_G4 = synth.BlockShape(hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=768, dtype="bf16")


def run_mfma(shape, n_layers, lens, steps, seed, sigma=0.05, check_kv=True):
    layers = [synth.layer_weights(shape, l, seed, sigma=sigma) for l in range(n_layers)]
    B, T = len(lens), sum(lens)
    cap = max(lens) + steps
    x = synth.hidden_states(T, shape, seed + 1)
    ost = orc.Stage(shape, layers, B, cap, "f32")
    gst = make_gpu_stage(shape, layers, B, cap, T)
    assert gst.uses_mfma()
    ref = ost.prefill(x, lens)
    got = to_host(gst.prefill(to_dev(x, "bf16"), lens))
    check(got, ref, x, "bf16", "prefill")
    if check_kv:
        for b in range(B):
            for l in {0, n_layers - 1}:
                k, v = gst.export_kv(l, b)
                assert rel_err(to_host(k), ost.K[l, b, :lens[b]]) <= TOL["bf16"], (b, l)
                assert rel_err(to_host(v), ost.V[l, b, :lens[b]]) <= TOL["bf16"], (b, l)
    for s in range(steps):
        xd = synth.hidden_states(B, shape, seed + 2 + s)
        ref = ost.decode_step(xd)
        got = to_host(gst.decode_step(to_dev(xd, "bf16")))
        check(got, ref, xd, "bf16", f"decode step {s}")
    if check_kv and steps:
        for b in range(B):
            k, v = gst.export_kv(n_layers - 1, b)
            n = lens[b] + steps
            assert rel_err(to_host(k), ost.K[n_layers - 1, b, :n]) <= TOL["bf16"]
            assert rel_err(to_host(v), ost.V[n_layers - 1, b, :n]) <= TOL["bf16"]
    return ost, gst


def test_mfma_single_request_one_layer():
    _, gst = run_mfma(SHAPE_G2, 1, [96], 3, 700)
    gst.destroy()


def test_mfma_ragged_batch_two_layers():
    # lengths: 1, not a multiple of 32, across a 64-row query tile, exact multiples
    _, gst = run_mfma(SHAPE_G2, 2, [1, 37, 130, 64, 257], 5, 701)
    gst.destroy()


def test_mfma_group_of_four_heads_and_tile_tails():
    # T' = 320+64 rows: one full 256-token GEMM tile and a partial one
    _, gst = run_mfma(SHAPE_G4, 2, [300, 33], 4, 702)
    gst.destroy()


def test_mfma_decode_across_chunk_and_block_boundaries():
    # context crosses a 32-key block (at 32/64) and the 256-key decode chunk
    _, gst = run_mfma(SHAPE_G2, 1, [250, 31], 12, 703)
    gst.destroy()


def test_mfma_matches_plain_kernels_closely():
    """Same stage through the shape-generic kernels: both sit within tolerance of the
    oracle, and within twice that of each other."""
    from paper_2511_14450_amd import binding
    shape = SHAPE_G2
    layers = [synth.layer_weights(shape, l, 704, sigma=0.05) for l in range(2)]
    lens = [70, 129]
    x = to_dev(synth.hidden_states(sum(lens), shape, 705), "bf16")
    a = make_gpu_stage(shape, layers, 2, 140, 199)
    b = make_gpu_stage(shape, layers, 2, 140, 199, flags=binding.HYP_FLAG_PLAIN_KERNELS)
    assert a.uses_mfma() and not b.uses_mfma()
    ya, yb = to_host(a.prefill(x, lens)), to_host(b.prefill(x, lens))
    assert rel_err(ya, yb) <= 2 * TOL["bf16"]
    a.destroy(); b.destroy()


def test_mfma_determinism_and_reprefill():
    import torch
    shape = SHAPE_G2
    layers = [synth.layer_weights(shape, 0, 706, sigma=0.05)]
    st = make_gpu_stage(shape, layers, 3, 200, 400)
    x1 = to_dev(synth.hidden_states(290, shape, 707), "bf16")
    y1 = st.prefill(x1, [160, 130]).clone()
    d1 = st.decode_step(x1[:2].contiguous()).clone()
    # a shorter prefill in between must not leave anything behind
    st.prefill(x1[:50].contiguous(), [20, 10, 20])
    st.decode_step(x1[:3].contiguous())
    y2 = st.prefill(x1, [160, 130])
    d2 = st.decode_step(x1[:2].contiguous())
    assert torch.equal(y1, y2) and torch.equal(d1, d2)
    st.destroy()


def test_decode_graph_replays_equal_kernel_by_kernel_launches():
    """The recorded decode-step graph is replayed many times, with prefill calls and
    synchronisations in between, and must give bit-identical results to launching
    the same kernels one by one."""
    import torch
    from paper_2511_14450_amd import binding
    shape = SHAPE_G2
    layers = [synth.layer_weights(shape, l, 708, sigma=0.05) for l in range(2)]
    lens = [40, 100, 7]
    x = to_dev(synth.hidden_states(sum(lens), shape, 709), "bf16")
    a = make_gpu_stage(shape, layers, 3, 200, 200)
    b = make_gpu_stage(shape, layers, 3, 200, 200, flags=binding.HYP_FLAG_NO_GRAPH)
    for rep in range(2):
        ya, yb = a.prefill(x, lens), b.prefill(x, lens)
        assert torch.equal(ya, yb)
        for s in range(6):
            xd = to_dev(synth.hidden_states(3, shape, 710 + s), "bf16")
            da, db = a.decode_step(xd), b.decode_step(xd)
            torch.cuda.synchronize()
            assert torch.equal(da, db), (rep, s)
        # a different batch size forces a new recording
        a.prefill(x[:47].contiguous(), [40, 7]); b.prefill(x[:47].contiguous(), [40, 7])
        xd = to_dev(synth.hidden_states(2, shape, 720), "bf16")
        assert torch.equal(a.decode_step(xd), b.decode_step(xd))
    a.destroy(); b.destroy()


def test_mfma_batch_32_and_single_token_prompts():
    # 32 resident requests (the widest decode block), among them 1-token prompts
    lens = [1, 2, 31, 32, 33, 63, 64, 65] + [5] * 24
    _, gst = run_mfma(SHAPE_G2, 1, lens, 3, 730, check_kv=False)
    gst.destroy()


@pytest.mark.parametrize("batch", [1, 3, 5, 9, 17, 31])
def test_mfma_decode_every_batch_width(batch):
    # the skinny GEMMs load activations only in the lanes of existing token columns: odd
    # and one-off widths around the 8 / 16 / 32 boundaries
    lens = [(7 * b) % 40 + 1 for b in range(batch)]
    _, gst = run_mfma(SHAPE_G4, 2, lens, 2, 740 + batch, check_kv=False)
    gst.destroy()


# hidden 5120 and FFN 7680 are the smallest widths here at which the skinny GEMMs of a decode step are
# split along K across workgroups (two slices for QKV and gate/up, three for the down projection)
SHAPE_SPLITK = synth.BlockShape(hidden=5120, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=7680, dtype="bf16")


@pytest.mark.parametrize("batch", [3, 17, 31])
def test_mfma_decode_split_k_at_odd_batch_widths(batch):
    # partial sums, arrival counters and the finishing workgroup's gather with 3, 17 and 31
    # live token columns (one, five and eight (token, row) pairs per finishing thread)
    lens = [(5 * b) % 9 + 1 for b in range(batch)]
    _, gst = run_mfma(SHAPE_SPLITK, 1, lens, 2, 760 + batch, sigma=0.02, check_kv=False)
    gst.destroy()


def test_mfma_split_k_decode_is_run_to_run_identical():
    # whichever workgroup of a row group arrives last adds the K slices in slice order:
    # eight repetitions of the same steps must agree bit for bit
    import torch
    shape = SHAPE_SPLITK
    layers = [synth.layer_weights(shape, 0, 770, sigma=0.02)]
    st = make_gpu_stage(shape, layers, 5, 64, 64)
    x = to_dev(synth.hidden_states(40, shape, 771), "bf16")
    xd = [to_dev(synth.hidden_states(5, shape, 772 + i), "bf16") for i in range(3)]
    ref = None
    for rep in range(8):
        st.prefill(x, [3, 11, 7, 9, 10])
        outs = [st.decode_step(d).clone() for d in xd]
        if ref is None:
            ref = outs
        else:
            assert all(torch.equal(a, b) for a, b in zip(ref, outs)), rep
    st.destroy()


def test_mfma_decode_fills_the_cache_to_capacity():
    """70 decode steps from a 58-token prompt: crosses two 32-key block boundaries and a
    decode chunk boundary and ends exactly at max_seq; one more step must be refused."""
    import paper_2511_14450_amd as hyp
    from paper_2511_14450_amd import binding
    ost, gst = run_mfma(SHAPE_G2, 1, [58, 3], 70, 731, check_kv=True)
    assert gst.context_len(0) == 128
    with pytest.raises(hyp.HypError) as e:
        gst.decode_step(to_dev(synth.hidden_states(2, SHAPE_G2, 999), "bf16"))
    assert e.value.status == binding.HYP_ECAPACITY
    gst.destroy()


def test_mfma_three_layer_stage_composition():
    # stage [0,3) == stage [0,1) then stage [1,3): the residual stream crosses stages as bf16
    shape = SHAPE_G2
    layers = [synth.layer_weights(shape, l, 732, sigma=0.05) for l in range(3)]
    lens = [90, 41]
    x = synth.hidden_states(sum(lens), shape, 733)
    ost = orc.Stage(shape, layers, 2, 140, "f32")
    ref = ost.prefill(x, lens)
    a = make_gpu_stage(shape, layers[:1], 2, 140, 131)
    b = make_gpu_stage(shape, layers[1:], 2, 140, 131, l_start=1)
    got = to_host(b.prefill(a.prefill(to_dev(x, "bf16"), lens), lens))
    check(got, ref, x, "bf16", "chained stages")
    a.destroy(); b.destroy()


def test_mfma_rms_eps_zero_with_padded_prompts():
    # eps = 0 is admitted: the rows that pad a prompt to a multiple of 64 have a zero sum of
    # squares and must not turn into 1/0 on their way into the caches
    shape = dataclasses.replace(SHAPE_G2, rms_eps=0.0)
    _, gst = run_mfma(shape, 2, [37, 130, 1], 3, 780)
    gst.destroy()
