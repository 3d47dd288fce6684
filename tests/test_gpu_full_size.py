"""Parity at the full Phi-3-medium block shape, in the launch configuration the
bench times (MFMA path, real widths, long and ragged contexts).  The oracle
cannot run 100+ TFLOP stages, so a one-block stage is checked on sampled rows:
the oracle forms keys and values for every position of a sampled request and
the complete block output for the sampled query rows (first, last, tile edges,
random), then follows with cached decode steps at the full context length."""
import numpy as np
import pytest

from oracle import hyp_oracle as orc
from workloads import synth
from tests.helpers import make_gpu_stage, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu
TOL = 2e-2
SHAPE = synth.PHI3_MEDIUM


@pytest.fixture(scope="module")
def phi3_layer():
    return synth.layer_weights(SHAPE, 0, synth.WORKLOADS["c3_stage10"].seed)


def sample_rows(L, rng, n_random=6):
    edges = [0, 1, 31, 32, 63, 64, 65, 127, 128, 255, 256, 257, L - 2, L - 1]
    rows = sorted({r for r in edges if 0 <= r < L} | {int(v) for v in rng.integers(0, L, n_random)})
    return rows


def check_requests(layer, lens, seed, sample_reqs, decode_steps, SHAPE=SHAPE, cap=None, paged=False):
    """`cap` = per-request capacity of the stage: it fixes the decode attention's chunking, so
    the tests of a bench workload pass the capacity the bench creates its stage with."""
    B, T = len(lens), sum(lens)
    cap = cap or max(lens) + decode_steps
    x = synth.hidden_states(T, SHAPE, seed)
    if paged:  # pages of 128 keys, handed to the requests in shuffled order
        from paper_2511_14450_amd import binding
        gst = make_gpu_stage(SHAPE, [layer], B, cap, T, flags=binding.HYP_FLAG_PAGED_KV)
        ppr = -(-((cap + 63) // 64 * 64) // 128)
        perm = np.random.default_rng(seed).permutation(B * ppr)
        gst.set_page_table([[int(v) for v in perm[r * ppr:(r + 1) * ppr]] for r in range(B)])
    else:
        gst = make_gpu_stage(SHAPE, [layer], B, cap, T)
    assert gst.uses_mfma()
    got = to_host(gst.prefill(to_dev(x, "bf16"), lens))
    starts = np.concatenate([[0], np.cumsum(lens)])
    rng = np.random.default_rng(seed)
    caches = {}
    worst = worst_update = 0.0
    for b in sample_reqs:
        L = lens[b]
        xb = x[starts[b]: starts[b] + L]
        rows = sample_rows(L, rng)
        Kc, Vc = orc.new_cache(SHAPE, L + decode_steps)
        ref = orc.layer_forward(SHAPE, layer, xb, 0, Kc, Vc, rows=rows)
        g = got[starts[b]: starts[b] + L][rows]
        e = rel_err(g, ref)
        eu = rel_err(g - xb[rows], ref - xb[rows])
        # the update (output - input) is held to the same bound, with no allowance for the bf16 rounding of the output
        assert e <= TOL and eu <= TOL, (b, e, eu)
        worst = max(worst, e)
        worst_update = max(worst_update, eu)
        # the cache the GPU built for this request, against the oracle's
        k, v = gst.export_kv(0, b)
        assert rel_err(to_host(k), Kc[:L]) <= TOL and rel_err(to_host(v), Vc[:L]) <= TOL
        caches[b] = (Kc, Vc)
    for s in range(decode_steps):
        xd = synth.hidden_states(B, SHAPE, seed + 100 + s)
        gd = to_host(gst.decode_step(to_dev(xd, "bf16")))
        for b in sample_reqs:
            Kc, Vc = caches[b]
            ref = orc.layer_forward(SHAPE, layer, xd[b: b + 1], lens[b] + s, Kc, Vc)
            e = rel_err(gd[b], ref[0])
            assert e <= TOL, (s, b, e)
            worst = max(worst, e)
    gst.destroy()
    print(f"\nlens {lens[:4]}{'...' if len(lens) > 4 else ''} cap {cap}: worst rel err {worst:.3e}, of the prefill update {worst_update:.3e}")
    return worst


def test_c2_layer_4x512_sampled_rows(phi3_layer):
    check_requests(phi3_layer, [512] * 4, 9100, sample_reqs=[0, 3], decode_steps=0)


def test_short_prompts_full_width_split_k_gemms(phi3_layer):
    # the paper's own request shape (Sec. V-A: 64-token prompts): one token tile, so the four
    # GEMMs have 20 - 140 output tiles and split their K loop across workgroups
    check_requests(phi3_layer, [64], 9150, sample_reqs=[0], decode_steps=1)
    check_requests(phi3_layer, [64, 17, 1], 9160, sample_reqs=[0, 1, 2], decode_steps=1)


def test_c3_layer_8x2048_sampled_rows_then_decode(phi3_layer):
    wl = synth.WORKLOADS["c3_stage10"]
    check_requests(phi3_layer, [2048] * 8, 9200, sample_reqs=[0, 5], decode_steps=2, cap=2048 + wl.decode_steps)


def test_c4_ragged_batch32_decode_at_long_context(phi3_layer):
    lens = synth.WORKLOADS["c4_decode_heavy"].lengths()
    assert len(lens) == 32 and min(lens) >= 1024 and max(lens) <= 4096
    longest, shortest = int(np.argmax(lens)), int(np.argmin(lens))
    check_requests(phi3_layer, lens, 9300, sample_reqs=[longest, shortest], decode_steps=2,
                   cap=max(lens) + synth.WORKLOADS["c4_decode_heavy"].decode_steps)


def test_c4_ragged_batch32_paged_cache_shuffled_table(phi3_layer):
    # the same workload with the cache in 128-key pages assigned in shuffled order
    lens = synth.WORKLOADS["c4_decode_heavy"].lengths()
    longest, shortest = int(np.argmax(lens)), int(np.argmin(lens))
    check_requests(phi3_layer, lens, 9350, sample_reqs=[longest, shortest], decode_steps=2,
                   cap=max(lens) + synth.WORKLOADS["c4_decode_heavy"].decode_steps, paged=True)


def test_c5_long_context_8192_sampled_rows_then_decode(phi3_layer):
    # one long request (the 8192-token prompts of the long-sequence workload) next to a short one
    check_requests(phi3_layer, [8192, 300], 9400, sample_reqs=[0, 1], decode_steps=2)


def test_c5_launch_shape_batch8_capacity_9216(phi3_layer):
    # the stage the long-sequence workload creates: 8 resident requests of capacity 8192 + 1024,
    # which makes the decode attention run 1024-key chunks, nine of them for the long request;
    # seven short requests keep the oracle's share affordable
    wl = synth.WORKLOADS["c5_long"]
    lens = [8192, 1, 31, 64, 100, 333, 1024, 1500]
    check_requests(phi3_layer, lens, 9450, sample_reqs=[0, 2, 7], decode_steps=2, cap=8192 + wl.decode_steps)


def test_three_blocks_at_full_width_whole_tensor():
    """A stage of three Phi-3-medium-shaped blocks over short prompts, every element against
    the oracle: inside a stage the down projection's residual epilogue hands its output and
    norm statistics straight to the next block's QKV projection (prefill and decode), which a
    one-block stage never exercises at widths 5120 / 17920."""
    seed = synth.WORKLOADS["c3_stage10"].seed
    layers = [synth.layer_weights(SHAPE, l, seed) for l in range(3)]
    lens, steps = [64, 17], 2
    x = synth.hidden_states(sum(lens), SHAPE, 9600)
    ost = orc.Stage(SHAPE, layers, 2, 80, "f32")
    gst = make_gpu_stage(SHAPE, layers, 2, 80, sum(lens))
    assert gst.uses_mfma()
    ref = ost.prefill(x, lens)
    got = to_host(gst.prefill(to_dev(x, "bf16"), lens))
    errs = [rel_err(got, ref), rel_err(got - x, ref - x)]
    for l in range(3):
        for b in range(2):
            k, v = gst.export_kv(l, b)
            errs += [rel_err(to_host(k), ost.K[l, b, :lens[b]]), rel_err(to_host(v), ost.V[l, b, :lens[b]])]
    for s in range(steps):
        xd = synth.hidden_states(2, SHAPE, 9601 + s)
        ref = ost.decode_step(xd)
        got = to_host(gst.decode_step(to_dev(xd, "bf16")))
        errs += [rel_err(got, ref), rel_err(got - xd, ref - xd)]
    gst.destroy()
    print(f"\nthree full-width blocks: prefill {errs[0]:.3e} (update {errs[1]:.3e}), worst of all {max(errs):.3e}")
    assert max(errs) <= TOL, errs


def test_llama3_8b_shaped_block_sampled_rows_then_decode():
    # the second model of Table I: hidden 4096, 32 query / 8 KV heads, FFN 14336
    shape = synth.LLAMA3_8B
    layer = synth.layer_weights(shape, 0, synth.WORKLOADS["n4_llama3_stage8"].seed)
    check_requests(layer, [2048, 777, 64], 9500, sample_reqs=[0, 1, 2], decode_steps=2, SHAPE=shape)
