"""Paged KV cache (HYP_FLAG_PAGED_KV): keys and values live in a pool of 128-key pages
addressed through a page table.  The block definition does not change, so the oracle is
the same plain-array cache; the tests shuffle the table, cross page boundaries while
decoding, compare with the contiguous layout bit for bit and exercise the table's rules."""
import numpy as np
import pytest

from oracle import hyp_oracle as orc
from workloads import synth
from tests.helpers import make_gpu_stage, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu
TOL = 2e-2
SHAPE = synth.BlockShape(hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=768, dtype="bf16")
PAGE = 128


def shuffled_table(batch, cap, seed, pool=None):
    ppr = -(-((cap + 63) // 64 * 64) // PAGE)
    pool = pool or batch * ppr
    perm = np.random.default_rng(seed).permutation(pool)[: batch * ppr]
    return [[int(v) for v in perm[r * ppr:(r + 1) * ppr]] for r in range(batch)]


def paged_stage(shape, layers, batch, cap, max_prefill, table=None, pool=0, flags=0):
    import paper_2511_14450_amd as hyp
    from paper_2511_14450_amd import binding
    cfg = hyp.stage_config(shape, batch, cap, max_prefill, flags=binding.HYP_FLAG_PAGED_KV | flags, kv_pool_pages=pool)
    dev = [{k: to_dev(v, shape.dtype) for k, v in w.items()} for w in layers]
    st = hyp.stage_create(cfg, 0, len(layers), dev)
    if table is not None:
        st.set_page_table(table)
    return st


def test_paged_shuffled_table_against_oracle_across_page_boundaries():
    # c4-style ragged batch; decode steps carry requests over the 128- and 256-key page edges
    lens, steps, seed = [120, 250, 5, 127, 383, 64], 12, 8500
    layers = [synth.layer_weights(SHAPE, l, seed, sigma=0.05) for l in range(3)]
    B, T, cap = len(lens), sum(lens), max(lens) + steps
    x = synth.hidden_states(T, SHAPE, seed + 1)
    ost = orc.Stage(SHAPE, layers, B, cap, "f32")
    gst = paged_stage(SHAPE, layers, B, cap, T, table=shuffled_table(B, cap, seed))
    assert gst.uses_mfma()
    ref = ost.prefill(x, lens)
    got = to_host(gst.prefill(to_dev(x, "bf16"), lens))
    errs = [rel_err(got, ref), rel_err(got - x, ref - x)]
    for s in range(steps):
        xd = synth.hidden_states(B, SHAPE, seed + 2 + s)
        ref = ost.decode_step(xd)
        got = to_host(gst.decode_step(to_dev(xd, "bf16")))
        errs += [rel_err(got, ref), rel_err(got - xd, ref - xd)]
    for l in (0, 2):
        for b in range(B):
            k, v = gst.export_kv(l, b)
            n = lens[b] + steps
            errs += [rel_err(to_host(k), ost.K[l, b, :n]), rel_err(to_host(v), ost.V[l, b, :n])]
    gst.destroy()
    print(f"\npaged, shuffled table: worst rel err {max(errs):.3e}")
    assert max(errs) <= TOL, errs


def test_paged_equals_contiguous_bit_for_bit():
    import torch
    lens, steps, seed = [300, 33, 129], 6, 8520
    layers = [synth.layer_weights(SHAPE, l, seed, sigma=0.05) for l in range(2)]
    B, T, cap = len(lens), sum(lens), max(lens) + steps + 1
    x = to_dev(synth.hidden_states(T, SHAPE, seed + 1), "bf16")
    slab = make_gpu_stage(SHAPE, layers, B, cap, T)
    ident = paged_stage(SHAPE, layers, B, cap, T)                                    # default table
    shuf = paged_stage(SHAPE, layers, B, cap, T, table=shuffled_table(B, cap, seed))
    ya = slab.prefill(x, lens)
    assert torch.equal(ya, ident.prefill(x, lens)) and torch.equal(ya, shuf.prefill(x, lens))
    for s in range(steps):
        xd = to_dev(synth.hidden_states(B, SHAPE, seed + 2 + s), "bf16")
        da = slab.decode_step(xd)
        assert torch.equal(da, ident.decode_step(xd)) and torch.equal(da, shuf.decode_step(xd)), s
    for b in range(B):
        (ka, va), (kb, vb) = slab.export_kv(1, b), shuf.export_kv(1, b)
        assert torch.equal(ka, kb) and torch.equal(va, vb)
    # the decode step for callers that cannot allocate reads the same table
    xd = to_dev(synth.hidden_states(B, SHAPE, seed + 50), "bf16")
    ya, yb = torch.empty_like(xd), torch.empty_like(xd)
    slab.decode_step(xd, ya); shuf.decode_step_noalloc(xd, yb)
    assert torch.equal(ya, yb)
    for st in (slab, ident, shuf):
        st.destroy()


def test_small_pool_and_table_rules():
    import paper_2511_14450_amd as hyp
    from paper_2511_14450_amd import binding
    seed = 8540
    layers = [synth.layer_weights(SHAPE, 0, seed, sigma=0.05)]
    # 4 slots of capacity 512 would need 16 pages; the pool has 6
    st = paged_stage(SHAPE, layers, 4, 512, 1024, pool=6)
    lens = [100, 130, 20]
    x = synth.hidden_states(sum(lens), SHAPE, seed + 1)
    with pytest.raises(hyp.HypError) as e:     # a small pool starts with no pages assigned
        st.prefill(to_dev(x, "bf16"), lens)
    assert e.value.status == binding.HYP_ECAPACITY
    for bad, status in (([[0, 1], [1, 2]], binding.HYP_EINVAL),       # page 1 twice
                        ([[0, 6]], binding.HYP_EINVAL),               # outside the pool
                        ([[0, 1, 2, 3, 4]], binding.HYP_ECAPACITY),   # beyond max_seq
                        ([[0]] * 5, binding.HYP_ECAPACITY)):          # more slots than max_batch
        with pytest.raises(hyp.HypError) as e:
            st.set_page_table(bad)
        assert e.value.status == status, bad
    st.set_page_table([[5, -1], [2, 0], [3, -1]])
    ost = orc.Stage(SHAPE, layers, 3, 512, "f32")
    assert rel_err(to_host(st.prefill(to_dev(x, "bf16"), lens)), ost.prefill(x, lens)) <= TOL
    # request 0 fills its only page after 28 steps; the 29th is refused and changes nothing
    for s in range(28):
        xd = synth.hidden_states(3, SHAPE, seed + 2 + s)
        ref = ost.decode_step(xd)
        got = to_host(st.decode_step(to_dev(xd, "bf16")))
        assert rel_err(got, ref) <= TOL, s
    xd = synth.hidden_states(3, SHAPE, seed + 40)
    with pytest.raises(hyp.HypError) as e:
        st.decode_step(to_dev(xd, "bf16"))
    assert e.value.status == binding.HYP_ECAPACITY and st.context_len(0) == 128
    with pytest.raises(hyp.HypError) as e:     # a page that holds cached keys may not move
        st.set_page_table([[4, 1], [2, 0], [3, -1]])
    assert e.value.status == binding.HYP_ESTATE
    st.set_page_table([[5, 1], [2, 0], [3, 4]])  # one more page for requests 0 and 2
    got = to_host(st.decode_step(to_dev(xd, "bf16")))
    assert rel_err(got, ost.decode_step(xd)) <= TOL
    k, v = st.export_kv(0, 0)
    assert rel_err(to_host(k), ost.K[0, 0, :129]) <= TOL and rel_err(to_host(v), ost.V[0, 0, :129]) <= TOL
    st.destroy()
    # the flag is refused where the MFMA kernels do not apply, and the table call without the flag
    with pytest.raises(hyp.HypError) as e:
        paged_stage(synth.TINY, [synth.layer_weights(synth.TINY, 0, 1)], 1, 16, 16)
    assert e.value.status == binding.HYP_ESHAPE
    plain = make_gpu_stage(SHAPE, layers, 1, 64, 64)
    with pytest.raises(hyp.HypError) as e:
        plain.set_page_table([[0]])
    assert e.value.status == binding.HYP_ESTATE
    plain.destroy()
