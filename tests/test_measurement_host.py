"""Host-side pieces of the measurement path (no GPU): kernel names of a rocprofv3 trace map to the kernel
classes bench.py reports, whatever their grid size; bench.py refuses more than one GPU with a message; the
committed HBM-traffic summary is only used for the kernel sources it was measured on."""
import json
import pathlib
import subprocess
import sys

import pytest

ROOT = pathlib.Path(__file__).resolve().parents[1]
sys.path.insert(0, str(ROOT))

from paper_2511_14450_amd import profile_summary as ps  # noqa: E402

NAMES = {
    "void hyp::(anonymous namespace)::k_gemm<2, 1>(hyp::(anonymous namespace)::GemmParams)": "gemm_qkv",
    "void hyp::(anonymous namespace)::k_gemm<3, 3>(hyp::(anonymous namespace)::GemmParams)": "gemm_o",
    "void hyp::(anonymous namespace)::k_gemm<1, 4>(hyp::(anonymous namespace)::GemmParams)": "gemm_gateup",
    "void hyp::(anonymous namespace)::k_gemm<3, 5>(hyp::(anonymous namespace)::GemmParams)": "gemm_down",
    "void hyp::(anonymous namespace)::k_gemm<0, 5>(hyp::(anonymous namespace)::GemmParams)": "gemm_down",
    "void hyp::(anonymous namespace)::k_dec_gemv<0, 2, 8, 6>(hyp::(anonymous namespace)::DecGemvParams)": "gemv_qkv",
    "void hyp::(anonymous namespace)::k_dec_gemv<2, 1, 4, 9>(hyp::(anonymous namespace)::DecGemvParams)": "gemv_o",
    "void hyp::(anonymous namespace)::k_dec_gemv<1, 2, 8, 10>(hyp::(anonymous namespace)::DecGemvParams)": "gemv_gateup",
    "void hyp::(anonymous namespace)::k_dec_gemv<2, 2, 8, 12>(hyp::(anonymous namespace)::DecGemvParams)": "gemv_down",
    "void hyp::(anonymous namespace)::k_dec_gemv<3, 2, 16, 12>(hyp::(anonymous namespace)::DecGemvParams)": "gemv_down",
    "void hyp::(anonymous namespace)::k_attn_prefill<4>(unsigned short const*, unsigned short const*)": "attn_prefill",
    "void hyp::(anonymous namespace)::k_attn_decode<2>(unsigned short const*)": "attn_decode",
    "hyp::(anonymous namespace)::k_attn_decode_merge(float const*, int const*, unsigned short*, int, int, int)": "attn_decode_merge",
    "void hyp::(anonymous namespace)::k_add_norm<0, 8>(unsigned short const*)": "add_norm",
    "hyp::(anonymous namespace)::k_rstd(float const*, float*, int const*, int, int, float)": "add_norm",
    "hyp::(anonymous namespace)::k_dec_begin(unsigned short const*)": "dec_begin",
}


@pytest.mark.parametrize("name", list(NAMES))
def test_trace_names_map_to_kernel_classes(name):
    assert ps.classify({"Kernel_Name": name}) == NAMES[name]


def test_every_gemm_class_of_the_header_is_known():
    import re
    header = (ROOT / "include" / "hyp_stage.h").read_text()
    ids = {m.group(1): int(m.group(2)) for m in re.finditer(r"HYP_K_(\w+) = (\d+)", header)}
    for key, cls in (("GEMM_QKV", "gemm_qkv"), ("GEMM_O", "gemm_o"), ("GEMM_GATEUP", "gemm_gateup"), ("GEMM_DOWN", "gemm_down"),
                     ("GEMV_QKV", "gemv_qkv"), ("GEMV_O", "gemv_o"), ("GEMV_GATEUP", "gemv_gateup"), ("GEMV_DOWN", "gemv_down")):
        assert ps.CLASS_BY_ID[ids[key]] == cls


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


def test_committed_traffic_is_tied_to_the_kernel_sources(tmp_path, monkeypatch):
    import bench
    f = pathlib.Path(bench.traffic_file("c5_long"))
    assert f.exists(), "profiles/ holds the traffic summary of the bench workload"
    d = json.loads(f.read_text())
    assert d["workload"] == "c5_long" and set(d["hbm_bytes_per_launch"]) >= {"gemv_gateup", "attn_decode", "gemm_gateup", "attn_prefill"}
    # a summary measured on other sources is not used
    g = tmp_path / "traffic_c5_long.json"
    g.write_text(json.dumps(dict(d, sources_sha256="0" * 64)))
    monkeypatch.setattr(bench, "traffic_file", lambda workload: str(g))
    assert bench.committed_traffic("c5_long") == {}
    # and one measured on these sources is
    g.write_text(json.dumps(dict(d, sources_sha256=bench.kernel_sources_digest())))
    assert bench.committed_traffic("c5_long") == d["hbm_bytes_per_launch"]
