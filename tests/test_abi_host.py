"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, sizes workspaces and rejects bad arguments
before touching the device."""
import ctypes as C
import pathlib
import re

import pytest

import paper_2511_14450_amd as hyp
from paper_2511_14450_amd import binding
from workloads import synth
from tests.helpers import make_config

ROOT = pathlib.Path(__file__).resolve().parents[1]


def test_library_exports_every_declared_symbol():
    header = (ROOT / "include" / "hyp_stage.h").read_text()
    declared = re.findall(r"HYP_API\s+[\w\s\*]+?\b(\w+)\s*\(", header)
    assert len(declared) >= 9
    lib = hyp.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert set(binding.EXPORTS) == set(declared)


def test_config_struct_matches_header_layout():
    # 12 x 4-byte fields with one 8-byte member aligned at offset 40
    assert C.sizeof(binding.StageConfig) == 56
    assert binding.StageConfig.max_prefill_tokens.offset == 40
    assert C.sizeof(binding.LayerWeights) == 9 * C.sizeof(C.c_void_p)


def test_workspace_bytes_scales_and_rejects():
    cfg = make_config(synth.TINY, 2, 128, 128)
    one = hyp.stage_workspace_bytes(cfg, 0, 1)
    two = hyp.stage_workspace_bytes(cfg, 3, 5)
    assert one > 0 and two > one
    per_layer = synth.TINY.params_per_layer() * 4
    assert two - one >= per_layer
    assert hyp.stage_workspace_bytes(cfg, 2, 2) == 0
    assert hyp.stage_workspace_bytes(cfg, -1, 2) == 0
    bad = make_config(synth.TINY, 2, 128, 128); bad.n_kv_heads = 3
    assert hyp.stage_workspace_bytes(bad, 0, 1) == 0
    assert "n_kv_heads" in hyp.stage_last_error(None)


def test_phi3_stage_fits_hbm():
    cfg = make_config(synth.PHI3_MEDIUM, 8, 8192 + 1024, 8 * 8192)
    need = hyp.stage_workspace_bytes(cfg, 0, 20)
    assert 0 < need < 200e9


@pytest.mark.parametrize("mutate,status", [
    (lambda c: setattr(c, "head_dim", 63), binding.HYP_ESHAPE),
    (lambda c: setattr(c, "n_kv_heads", 3), binding.HYP_ESHAPE),
    (lambda c: setattr(c, "hidden", 0), binding.HYP_ESHAPE),
    (lambda c: setattr(c, "dtype", 7), binding.HYP_EINVAL),
    (lambda c: setattr(c, "kv_pool_pages", 1), binding.HYP_EINVAL),   # only with HYP_FLAG_PAGED_KV
    (lambda c: setattr(c, "flags", 64), binding.HYP_EINVAL),
])
def test_create_rejects_bad_config_without_device(mutate, status):
    lib = hyp.load_library()
    cfg = make_config(synth.TINY, 1, 64, 64)
    mutate(cfg)
    layers = (binding.LayerWeights * 1)()
    out = C.c_void_p()
    rc = lib.stage_create(C.byref(cfg), 0, 1, layers, None, 0, None, C.byref(out))
    assert rc == status and not out.value
    assert hyp.stage_last_error(None)


def test_null_and_range_arguments():
    lib = hyp.load_library()
    cfg = make_config(synth.TINY, 1, 64, 64)
    layers = (binding.LayerWeights * 1)()
    out = C.c_void_p()
    assert lib.stage_create(None, 0, 1, layers, None, 0, None, C.byref(out)) == binding.HYP_EINVAL
    assert lib.stage_create(C.byref(cfg), 1, 1, layers, None, 0, None, C.byref(out)) == binding.HYP_EINVAL
    assert lib.stage_create(C.byref(cfg), 0, 1, layers, None, 0, None, C.byref(out)) == binding.HYP_EINVAL  # workspace NULL
    assert lib.stage_prefill(None, None, None, 1, None) == binding.HYP_EINVAL
    assert lib.stage_decode_step(None, None, None) == binding.HYP_EINVAL
    assert lib.stage_destroy(None) == binding.HYP_EINVAL
    assert lib.stage_uses_mfma(None) == 0


def test_foreign_handles_are_refused_not_dereferenced():
    # every entry point looks its handle up among the live stages first: a pointer the library
    # never handed out (or one it already destroyed) is HYP_EINVAL
    lib = hyp.load_library()
    junk = C.create_string_buffer(4096)
    h = C.c_void_p(C.addressof(junk))
    assert lib.stage_destroy(h) == binding.HYP_EINVAL
    assert lib.stage_decode_step(h, h, h) == binding.HYP_EINVAL
    assert lib.stage_decode_step_noalloc(h, h, h) == binding.HYP_EINVAL
    assert lib.stage_prefill(h, h, None, 1, h) == binding.HYP_EINVAL
    assert lib.stage_export_kv(h, 0, 0, h, h) == binding.HYP_EINVAL
    n = C.c_int32()
    assert lib.stage_context_len(h, 0, C.byref(n)) == binding.HYP_EINVAL
    assert lib.stage_profile(h, 0) == binding.HYP_EINVAL
    assert lib.stage_uses_mfma(h) == 0
    assert b"live" in lib.stage_last_error(h)
