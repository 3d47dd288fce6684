"""stage_decode_step_noalloc (the decode step for callers that cannot allocate) against
stage_decode_step, through the C ABI: the same kernels with their temporaries in the
library's static device array must give the same bits.  Two calls in a row share the array,
the second on a smaller batch; then a stage whose temporaries exceed the array is refused."""
import ctypes as C

import numpy as np
import pytest

from workloads import synth
from tests.helpers import make_config, make_gpu_stage, to_dev

pytestmark = pytest.mark.gpu

# at these widths the skinny GEMMs are split along K, so partial sums and arrival counters are in use
SHAPE = synth.BlockShape(hidden=5120, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=7680, dtype="bf16")


def _decode_raw(lib, entry, stage, x, y):
    rc = getattr(lib, entry)(stage.handle, C.c_void_p(x.data_ptr()), C.c_void_p(y.data_ptr()))
    assert rc == 0, (entry, rc, lib.stage_last_error(stage.handle))


def test_noalloc_decode_equals_regular_decode_on_consecutive_calls():
    import torch
    import paper_2511_14450_amd as hyp
    lib = hyp.load_library()
    layers = [synth.layer_weights(SHAPE, l, 8300, sigma=0.02) for l in range(2)]
    ref = make_gpu_stage(SHAPE, layers, 5, 300, 600)
    new = make_gpu_stage(SHAPE, layers, 5, 300, 600)
    assert ref.uses_mfma() and new.uses_mfma()
    # first call: batch 5 with contexts across a decode chunk; second call: batch 2, short contexts
    for call, lens in enumerate(([3, 270, 7, 64, 10], [33, 5])):
        x = to_dev(synth.hidden_states(sum(lens), SHAPE, 8301 + call), "bf16")
        assert torch.equal(ref.prefill(x, lens), new.prefill(x, lens))
        for s in range(3):
            xd = to_dev(synth.hidden_states(len(lens), SHAPE, 8310 + 10 * call + s), "bf16")
            ya, yb = torch.empty_like(xd), torch.full_like(xd, float("nan"))
            _decode_raw(lib, "stage_decode_step", ref, xd, ya)
            _decode_raw(lib, "stage_decode_step_noalloc", new, xd, yb)
            torch.cuda.synchronize()
            assert torch.equal(ya, yb), (call, s)
        for b in range(len(lens)):
            assert ref.context_len(b) == new.context_len(b) == lens[b] + 3
            (ka, va), (kb, vb) = ref.export_kv(1, b), new.export_kv(1, b)
            assert torch.equal(ka, kb) and torch.equal(va, vb)
    # the two entry points may alternate on one stage
    xd = to_dev(synth.hidden_states(2, SHAPE, 8340), "bf16")
    ya, yb = torch.empty_like(xd), torch.empty_like(xd)
    _decode_raw(lib, "stage_decode_step_noalloc", ref, xd, ya)
    _decode_raw(lib, "stage_decode_step", new, xd, yb)
    torch.cuda.synchronize()
    assert torch.equal(ya, yb)
    ref.destroy(); new.destroy()


def test_noalloc_decode_refuses_what_does_not_fit_or_does_not_apply():
    import torch
    import paper_2511_14450_amd as hyp
    from paper_2511_14450_amd import binding
    lib = hyp.load_library()
    # an FFN of 131072 features: the gate/up GEMV's room for partial sums, 2 x 131072 rows x 32 tokens x 4 B,
    # alone passes 32 MiB; zero weights are enough, the stage is never run
    big = synth.BlockShape(hidden=2048, n_q_heads=16, n_kv_heads=4, head_dim=128, ffn_dim=131072, dtype="bf16")
    w = {n: torch.zeros(shp, dtype=torch.bfloat16, device="cuda") for n, shp in big.weight_shapes().items()}
    st = hyp.stage_create(make_config(big, 8, 128, 128), 0, 1, [w])
    x = torch.zeros((8, big.hidden), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(hyp.HypError) as e:
        st.decode_step_noalloc(x, torch.empty_like(x))
    assert e.value.status == binding.HYP_ECAPACITY and "static array" in str(e.value)
    st.destroy()
    # an fp32 stage runs the shape-generic kernels
    tiny = make_gpu_stage(synth.TINY, [synth.layer_weights(synth.TINY, 0, 1)], 1, 16, 16)
    xt = to_dev(synth.hidden_states(4, synth.TINY, 2), "f32")
    tiny.prefill(xt, [4])
    with pytest.raises(hyp.HypError) as e:
        tiny.decode_step_noalloc(xt[:1].contiguous(), torch.empty_like(xt[:1]))
    assert e.value.status == binding.HYP_ESHAPE
    tiny.destroy()
