"""Seeded random sweep over what the fixed parity cases leave between them: head groupings
(1 - 4 query heads per KV head), widths, stage depths, batch widths up to 32, prompt
lengths on and off the 32 / 64 / 128 boundaries, slab and shuffled-page caches, capacity
with and without slack.  Every case runs the MFMA stage through the C ABI against the CPU
oracle (Sec. III-A block, Eq. 1 stacking), whole tensors, prefill + decode steps, 2e-2."""
import os

import numpy as np
import pytest

from oracle import hyp_oracle as orc
from workloads import synth
from tests.helpers import make_gpu_stage, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu
TOL = 2e-2
N_CASES = int(os.environ.get("HYP_RANDOM_CASES", "24"))  # more seeds for a longer sweep


def draw_case(i):
    rng = np.random.default_rng(77_000 + i)
    n_kv = int(rng.choice([2, 4]))
    G = int(rng.choice([1, 2, 3, 4]))
    hidden = int(rng.choice([256, 512, 768]))
    ffn = int(rng.choice([256, 512, 768, 1280]))
    shape = synth.BlockShape(hidden=hidden, n_q_heads=G * n_kv, n_kv_heads=n_kv, head_dim=128, ffn_dim=ffn, dtype="bf16")
    n_layers = int(rng.integers(1, 4))
    batch = int(rng.choice([1, 2, 3, 5, 8, 13, 32]))
    edges = [1, 31, 32, 33, 63, 64, 65, 127, 128, 129]
    lens = [int(rng.choice(edges)) if rng.random() < 0.4 else int(rng.integers(1, 200)) for _ in range(batch)]
    steps = int(rng.integers(1, 6))
    paged = bool(rng.random() < 0.5)
    slack = int(rng.choice([0, 1, 70]))
    return shape, n_layers, lens, steps, paged, slack


@pytest.mark.parametrize("i", range(N_CASES))
def test_random_case_against_oracle(i):
    from paper_2511_14450_amd import binding
    shape, n_layers, lens, steps, paged, slack = draw_case(i)
    seed = 78_000 + 10 * i
    # N(0, 0.05^2) projections: sub-layer updates of the size N(0, 0.02^2) gives at hidden 5120
    layers = [synth.layer_weights(shape, l, seed, sigma=0.05) for l in range(n_layers)]
    B, T = len(lens), sum(lens)
    cap = max(lens) + steps + slack
    x = synth.hidden_states(T, shape, seed + 1)
    ost = orc.Stage(shape, layers, B, cap, "f32")
    gst = make_gpu_stage(shape, layers, B, cap, T, flags=binding.HYP_FLAG_PAGED_KV if paged else 0)
    assert gst.uses_mfma()
    if paged:
        ppr = -(-((cap + 63) // 64 * 64) // binding.HYP_KV_PAGE_KEYS)
        perm = np.random.default_rng(seed + 2).permutation(B * ppr)
        gst.set_page_table([[int(v) for v in perm[r * ppr:(r + 1) * ppr]] for r in range(B)])
    what = f"case {i}: heads {shape.n_q_heads}/{shape.n_kv_heads} hidden {shape.hidden} ffn {shape.ffn_dim} " \
           f"blocks {n_layers} lens {lens[:6]}{'...' if B > 6 else ''} steps {steps} paged {paged} cap {cap}"
    print("\n" + what, flush=True)
    ref = ost.prefill(x, lens)
    got = to_host(gst.prefill(to_dev(x, "bf16"), lens))
    worst = max(rel_err(got, ref), rel_err(got - x, ref - x))
    assert worst <= TOL, (what, "prefill", worst)
    for s in range(steps):
        xd = synth.hidden_states(B, shape, seed + 3 + s)
        ref = ost.decode_step(xd)
        got = to_host(gst.decode_step(to_dev(xd, "bf16")))
        e = max(rel_err(got, ref), rel_err(got - xd, ref - xd))
        assert e <= TOL, (what, f"decode step {s}", e)
        worst = max(worst, e)
    for b in {0, B - 1}:
        k, v = gst.export_kv(n_layers - 1, b)
        n = lens[b] + steps
        e = max(rel_err(to_host(k), ost.K[n_layers - 1, b, :n]), rel_err(to_host(v), ost.V[n_layers - 1, b, :n]))
        assert e <= TOL, (what, f"cache of request {b}", e)
        worst = max(worst, e)
    assert gst.context_len(0) == lens[0] + steps
    gst.destroy()
    print(f"worst rel err {worst:.3e}", flush=True)


N_MEDIUM = int(os.environ.get("HYP_RANDOM_MEDIUM_CASES", "4"))


def draw_medium_case(i):
    """One block, wide enough and with enough tokens that the projections have 60 .. 1500 output tiles:
    on both sides of where the GEMMs stop splitting their K loop, whole and partly filled rounds of
    256 workgroups, ragged last token tiles."""
    rng = np.random.default_rng(79_000 + i)
    n_kv = int(rng.choice([2, 4, 8]))
    G = int(rng.choice([1, 2, 4]))
    hidden = int(rng.choice([1024, 1536, 2048]))
    ffn = int(rng.choice([1024, 2816, 4096]))
    shape = synth.BlockShape(hidden=hidden, n_q_heads=G * n_kv, n_kv_heads=n_kv, head_dim=128, ffn_dim=ffn, dtype="bf16")
    batch = int(rng.choice([1, 3, 8, 20]))
    total = int(rng.integers(1500, 9000))
    cuts = np.sort(rng.integers(1, total, size=batch - 1)) if batch > 1 else np.array([], dtype=np.int64)
    lens = [int(v) for v in np.diff(np.concatenate([[0], cuts, [total]])) if v > 0]
    return shape, lens, int(rng.integers(1, 4)), bool(rng.random() < 0.5)


@pytest.mark.parametrize("i", range(N_MEDIUM))
def test_random_medium_case_against_oracle(i):
    from paper_2511_14450_amd import binding
    shape, lens, steps, paged = draw_medium_case(i)
    seed = 80_000 + 10 * i
    layers = [synth.layer_weights(shape, 0, seed, sigma=0.03)]
    B, T = len(lens), sum(lens)
    cap = max(lens) + steps
    x = synth.hidden_states(T, shape, seed + 1)
    ost = orc.Stage(shape, layers, B, cap, "f32")
    gst = make_gpu_stage(shape, layers, B, cap, T, flags=binding.HYP_FLAG_PAGED_KV if paged else 0)
    assert gst.uses_mfma()
    what = f"medium case {i}: heads {shape.n_q_heads}/{shape.n_kv_heads} hidden {shape.hidden} ffn {shape.ffn_dim} " \
           f"tokens {T} in {B} requests (longest {max(lens)}) steps {steps} paged {paged}"
    print("\n" + what, flush=True)
    ref = ost.prefill(x, lens)
    got = to_host(gst.prefill(to_dev(x, "bf16"), lens))
    worst = max(rel_err(got, ref), rel_err(got - x, ref - x))
    assert worst <= TOL, (what, "prefill", worst)
    for s in range(steps):
        xd = synth.hidden_states(B, shape, seed + 3 + s)
        ref = ost.decode_step(xd)
        got = to_host(gst.decode_step(to_dev(xd, "bf16")))
        e = max(rel_err(got, ref), rel_err(got - xd, ref - xd))
        assert e <= TOL, (what, f"decode step {s}", e)
        worst = max(worst, e)
    b = int(np.argmax(lens))
    k, v = gst.export_kv(0, b)
    n = lens[b] + steps
    e = max(rel_err(to_host(k), ost.K[0, b, :n]), rel_err(to_host(v), ost.V[0, b, :n]))
    assert e <= TOL, (what, "cache of the longest request", e)
    gst.destroy()
    print(f"worst rel err {max(worst, e):.3e}", flush=True)
