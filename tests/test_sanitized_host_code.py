"""The host-only code under AddressSanitizer and UndefinedBehaviorSanitizer: the planner
(csrc/planner.hip holds no device code and compiles as plain C++) and the C oracle are built
with -fsanitize=address,undefined into one driver program, fed seeded cases, and must
(a) finish without a sanitizer report and (b) print exactly what the regular builds return
(the planner against the Python oracle of Algorithms 1 and 2, the C oracle against its own
unsanitized build)."""
import os
import pathlib
import shutil
import struct
import subprocess

import numpy as np
import pytest

from oracle import hyp_oracle as orc
from oracle import hyperion_plan as oplan
from workloads import synth

ROOT = pathlib.Path(__file__).resolve().parents[1]
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-O1", "-g"]


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    if not shutil.which("g++"):
        pytest.skip("no host compiler")
    d = tmp_path_factory.mktemp("san")
    inc = f"-I{ROOT / 'include'}"
    steps = [
        ["g++", "-std=c++17", *SAN, inc, "-x", "c++", "-c", str(ROOT / "paper_2511_14450_amd/csrc/planner.hip"), "-o", str(d / "planner.o")],
        ["gcc", "-std=c11", "-fopenmp", *SAN, "-c", str(ROOT / "oracle/hyp_oracle.c"), "-o", str(d / "oracle.o")],
        ["g++", "-std=c++17", *SAN, inc, "-c", str(ROOT / "tests/sanitize/san_driver.cpp"), "-o", str(d / "driver.o")],
        ["g++", "-fsanitize=address,undefined", "-fopenmp", str(d / "planner.o"), str(d / "oracle.o"), str(d / "driver.o"),
         "-o", str(d / "san_driver"), "-lm"],
    ]
    for cmd in steps:
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
    return d / "san_driver"


def run_driver(driver, text):
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="4")
    r = subprocess.run([str(driver)], input=text, capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
    return r.stdout.splitlines()


def fmt(v):
    return " ".join(repr(float(x)) for x in v)


def test_planner_under_sanitizers_matches_the_oracle(driver):
    rng = np.random.default_rng(31337)
    cases, expect = [], []
    for i in range(40):
        T = int(rng.integers(1, 6))
        N = int(rng.integers(T, 40))
        f = rng.uniform(0.0, 3.0, N).round(3); m = rng.uniform(0.0, 2.0, N).round(3)
        if i % 7 == 0:
            f[rng.integers(0, N)] = 0.0
        C = rng.uniform(0.5, 4.0, T).round(3)
        M = rng.uniform(0.3, 1.5, T).round(3) * m.sum() / T * (0.6 if i % 5 == 0 else 2.0)
        eps = 1e-6
        cases.append(f"split {N} {T} {eps!r}\n{fmt(f)}\n{fmt(m)}\n{fmt(C)}\n{fmt(M)}\n")
        p, tau = oplan.hypsplit_dp(list(map(float, f)), list(map(float, m)), list(map(float, C)), list(map(float, M)), eps)
        expect.append(("split", p, tau))
    for i in range(30):
        K = int(rng.integers(1, 7))
        C = rng.uniform(0.5, 3.0, K).round(2); Ma = rng.uniform(0.0, 2.0, K).round(2)
        av = rng.integers(0, 2, K); Fr = rng.uniform(0, 2, K).round(2); Fw = rng.uniform(0, 2, K).round(2)
        cases.append(f"sched {K} 1.25 1.0\n{fmt(C)}\n{fmt(Ma)}\n{fmt(av)}\n{fmt(Fr)}\n{fmt(Fw)}\n")
        expect.append(("sched", oplan.hypsched_rt(1.25, 1.0, list(C), list(Ma), [bool(a) for a in av], list(Fr), list(Fw))))
    for i in range(8):
        T = int(rng.integers(1, 4)); n = int(rng.integers(1, 40))
        nodes = [int(v) for v in rng.integers(1, 4, T)]
        arr = np.sort(rng.exponential(1.0 / 0.7, n).cumsum()).round(4)
        F = rng.uniform(0.5, 2.0, T).round(3); ma = rng.uniform(0.1, 1.0, T).round(3)
        C = [list(rng.uniform(0.5, 2.0, k).round(3)) for k in nodes]
        M = [list(rng.uniform(0.8, 3.0, k).round(3)) for k in nodes]
        tr = rng.uniform(0.0, 0.3, max(T - 1, 0)).round(3)
        flat = lambda xs: [x for c in xs for x in c]
        cases.append(f"sim {n} {T} 0\n{fmt(arr)}\n{fmt(F)}\n{fmt(ma)}\n{fmt(nodes)}\n{fmt(flat(C))}\n{fmt(flat(M))}\n{fmt(tr)}\n")
        expect.append(("sim", oplan.simulate_tiers(list(map(float, arr)), list(map(float, F)), list(map(float, ma)), C, M,
                                                   list(map(float, tr)))))
    lines = run_driver(driver, "".join(cases))
    assert len(lines) == len(expect)
    for line, exp in zip(lines, expect):
        tok = line.split()
        assert tok[0] == exp[0] and int(tok[1]) == 0, line
        if exp[0] == "split":
            _, p, tau = exp
            assert int(tok[2]) == (0 if p is None else 1)
            assert float(tok[3]) == tau
            assert [int(v) for v in tok[4:]] == (p or [])
        elif exp[0] == "sched":
            assert int(tok[2]) == (-1 if exp[1] is None else exp[1])
        else:
            node, fin = exp[1]
            got = tok[2:]
            flat_node = [k if k is not None else -1 for q in node for k in q]
            flat_fin = [t for q in fin for t in q]
            assert [int(v) for v in got[0::2]] == flat_node
            assert [float(v) for v in got[1::2]] == flat_fin


def test_c_oracle_under_sanitizers_matches_its_regular_build(driver, tmp_path):
    # head_dim 10 and widths that are multiples of nothing: every loop bound is exercised
    shape = synth.BlockShape(hidden=36, n_q_heads=6, n_kv_heads=3, head_dim=10, ffn_dim=50, dtype="f32")
    n_layers, lens, steps = 2, [5, 1, 9], 3
    layers = [synth.layer_weights(shape, l, 41, sigma=0.1) for l in range(n_layers)]
    x = synth.hidden_states(sum(lens), shape, 42)
    xd = np.stack([synth.hidden_states(len(lens), shape, 43 + s) for s in range(steps)])
    blob = struct.pack("<8i2d", shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn_dim,
                       n_layers, len(lens), steps, shape.rms_eps, shape.rope_base)
    blob += np.asarray(lens, dtype=np.int32).tobytes()
    for w in layers:
        for name in synth.WEIGHT_NAMES:
            blob += np.ascontiguousarray(w[name], dtype=np.float32).tobytes()
    blob += np.ascontiguousarray(x, dtype=np.float32).tobytes() + np.ascontiguousarray(xd, dtype=np.float32).tobytes()
    path = tmp_path / "stage.bin"
    path.write_bytes(blob)
    lines = run_driver(driver, f"stage {path}\n")
    assert len(lines) == 1 + steps
    ost = orc.Stage(shape, layers, len(lens), max(lens) + steps, "f32")
    ref = [ost.prefill(x, lens)] + [ost.decode_step(xd[s]) for s in range(steps)]
    for line, r in zip(lines, ref):
        got = np.array([float(v) for v in line.split()[2:]], dtype=np.float32)
        assert np.array_equal(got, r.reshape(-1).astype(np.float32))  # %.9g round-trips float32
