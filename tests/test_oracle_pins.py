"""Pins of the CPU oracle against things other than itself: hand-derived closed
forms (tests/golden/closed_forms.json), invariants of the definitions, library
routines in float64, and a second evaluation written with an explicit mask
matrix.  A dropped term, a wrong sign or index or a transposed operand in
oracle/hyp_oracle.c fails at least one of these."""
import dataclasses
import json
import pathlib

import numpy as np
import pytest

from oracle import hyp_oracle as orc
from workloads import synth

GOLD = json.loads((pathlib.Path(__file__).parent / "golden" / "closed_forms.json").read_text())
REALS = ("f32", "f64")
TOL = {"f32": 2e-6, "f64": 1e-13}


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ linear
@pytest.mark.parametrize("real", REALS)
def test_linear_matches_float64_matmul(real):
    g = rng(1)
    for (T, K, N) in [(1, 7, 5), (5, 33, 9), (17, 256, 40)]:
        x = g.standard_normal((T, K)); W = g.standard_normal((N, K))
        ref = x.astype(np.float64) @ W.astype(np.float64).T
        got = orc.linear(x, W, real)
        assert got.shape == (T, N)
        assert np.abs(got - ref).max() / np.abs(ref).max() < (1e-5 if real == "f32" else 1e-13)


# ------------------------------------------------------------------ RMSNorm
@pytest.mark.parametrize("real", REALS)
def test_rmsnorm_closed_forms(real):
    c = GOLD["rmsnorm_3_4"]
    y = orc.rmsnorm(np.array([c["x"]]), np.array(c["g"]), 0.0, real)
    assert np.allclose(y[0], c["out"], rtol=TOL[real] * 10, atol=0)
    g = rng(2)
    x = g.standard_normal((6, 96))
    y = orc.rmsnorm(x, np.ones(96), 0.0, real)
    assert np.allclose((y.astype(np.float64) ** 2).mean(axis=1), 1.0, atol=1e-5)
    # scale invariance (eps = 0) and constant rows
    y2 = orc.rmsnorm(3.7 * x, np.ones(96), 0.0, real)
    assert np.allclose(y, y2, atol=1e-5)
    gain = g.standard_normal(96)
    yc = orc.rmsnorm(np.full((1, 96), -2.5), gain, 0.0, real)
    assert np.allclose(yc[0], -gain, atol=1e-5)
    # eps sits inside the square root, added to the mean square
    ye = orc.rmsnorm(np.full((1, 4), 2.0), np.ones(4), 5.0, real)
    assert np.allclose(ye[0], 2.0 / 3.0, atol=1e-6)


# ------------------------------------------------------------------ RoPE
@pytest.mark.parametrize("real", REALS)
def test_rope_golden_and_invariants(real):
    c = GOLD["rope_unit_vector"]
    z = np.array(c["z"]).reshape(1, 1, 4)
    out = orc.rope(z, [c["pos"]], 10000.0, real)
    assert np.allclose(out.ravel(), c["out"], atol=TOL[real] * 4)
    g = rng(3)
    d, nh, T = 16, 3, 5
    z = g.standard_normal((T, nh, d))
    pos = np.array([0, 1, 7, 100, 4095])
    r = orc.rope(z, pos, 10000.0, real).astype(np.float64)
    # position 0 is the identity
    assert np.allclose(r[0], z[0], atol=1e-6)
    # each (i, i+d/2) pair keeps its norm
    n0 = z[..., : d // 2] ** 2 + z[..., d // 2:] ** 2
    n1 = r[..., : d // 2] ** 2 + r[..., d // 2:] ** 2
    assert np.allclose(n0, n1, rtol=1e-5)
    # pair i turns by exactly pos * base^(-2i/d) in the counter-clockwise sense
    for t in range(T):
        for i in range(d // 2):
            ang = pos[t] * 10000.0 ** (-2.0 * i / d)
            a, b = z[t, 0, i], z[t, 0, i + d // 2]
            assert np.isclose(r[t, 0, i], a * np.cos(ang) - b * np.sin(ang), atol=2e-5)
            assert np.isclose(r[t, 0, i + d // 2], b * np.cos(ang) + a * np.sin(ang), atol=2e-5)


@pytest.mark.parametrize("real", REALS)
def test_rope_inner_product_depends_on_offset_only(real):
    g = rng(4)
    d = 32
    q = g.standard_normal((1, 1, d)); k = g.standard_normal((1, 1, d))
    def ip(m, n):
        return float((orc.rope(q, [m], 10000.0, real).astype(np.float64)
                      * orc.rope(k, [n], 10000.0, real).astype(np.float64)).sum())
    base = ip(13, 5)
    for shift in (1, 1000, 8000):
        assert abs(ip(13 + shift, 5 + shift) - base) < (2e-5 if real == "f32" else 1e-10) * (1 + abs(base))
    assert abs(ip(14, 5) - base) > 1e-3  # and it does depend on the offset


# ------------------------------------------------------------------ softmax
@pytest.mark.parametrize("real", REALS)
def test_softmax_rows(real):
    g = rng(5)
    for n in (1, 2, 17, 300):
        s = g.standard_normal(n) * 5
        p = orc.softmax(s, real).astype(np.float64)
        assert abs(p.sum() - 1) < 1e-6 and (p >= 0).all()
        assert np.allclose(p, orc.softmax(s + 123.0, real), atol=2e-5 if real == "f32" else 1e-12)
        e = np.exp(s - s.max())
        assert np.allclose(p, e / e.sum(), atol=1e-6)
    # large scores do not overflow
    p = orc.softmax(np.array([1e4, 1e4 - np.log(3.0)]), real)
    assert np.allclose(p, [0.75, 0.25], atol=1e-3 if real == "f32" else 1e-9)


# ------------------------------------------------------------------ attention
def attention_mask_matrix_f64(q, q_pos, K, V):
    """Second evaluation straight from the definition, float64, with an explicit
    additive mask matrix and repeated KV heads (written without reference to the
    C code: einsum over a dense [heads, rows, keys] tensor)."""
    q = q.astype(np.float64); K = K.astype(np.float64); V = V.astype(np.float64)
    R, nq, d = q.shape
    nk, nkv, _ = K.shape
    rep = nq // nkv
    Kf = np.repeat(K, rep, axis=1)
    Vf = np.repeat(V, rep, axis=1)
    s = np.einsum("rhd,jhd->hrj", q, Kf) / np.sqrt(d)
    mask = np.where(np.arange(nk)[None, :] <= np.asarray(q_pos)[:, None], 0.0, -np.inf)
    s = s + mask[None]
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    return np.einsum("hrj,jhd->rhd", p, Vf), p


@pytest.mark.parametrize("real", REALS)
def test_attention_golden_two_keys(real):
    c = GOLD["attention_two_keys"]
    q = np.array(c["q"]).reshape(1, 1, 4)
    K = np.array(c["k"]).reshape(2, 1, 4); V = np.array(c["v"]).reshape(2, 1, 4)
    out, p = orc.attention(q, [1], K, V, real, return_probs=True)
    assert np.allclose(p[0, 0], c["probs"], atol=1e-6)
    assert np.allclose(out[0, 0], c["out"], atol=1e-6)
    # with the second key masked (query at position 0) the output is v0
    out0 = orc.attention(q, [0], K, V, real)
    assert np.allclose(out0[0, 0], c["v"][0], atol=1e-7)


@pytest.mark.parametrize("real", REALS)
def test_attention_bruteforce_tiny(real):
    g = rng(6)
    for (S, nq, nkv, d) in [(1, 1, 1, 2), (5, 2, 1, 4), (8, 4, 2, 4), (7, 6, 3, 2), (8, 4, 4, 4)]:
        q = g.standard_normal((S, nq, d)) * 2
        K = g.standard_normal((S, nkv, d)) * 2
        V = g.standard_normal((S, nkv, d))
        pos = np.arange(S)
        ref, pref = attention_mask_matrix_f64(q, pos, K, V)
        out, p = orc.attention(q, pos, K, V, real, return_probs=True)
        assert np.abs(out - ref).max() < (5e-6 if real == "f32" else 1e-12)
        assert np.abs(p - pref).max() < (5e-6 if real == "f32" else 1e-12)
        # softmax rows sum to one over the visible prefix and are zero beyond it
        assert np.allclose(p.sum(axis=-1), 1.0, atol=1e-6)
        assert (np.triu(p, k=1) == 0).all()
    # rows at arbitrary positions against a longer cache (decode-like)
    q = g.standard_normal((3, 4, 4)); K = g.standard_normal((9, 2, 4)); V = g.standard_normal((9, 2, 4))
    pos = np.array([8, 2, 5])
    ref, _ = attention_mask_matrix_f64(q, pos, K, V)
    assert np.abs(orc.attention(q, pos, K, V, real) - ref).max() < (5e-6 if real == "f32" else 1e-12)


@pytest.mark.parametrize("real", REALS)
def test_attention_special_cases(real):
    g = rng(7)
    S, nq, nkv, d = 6, 4, 2, 8
    q = g.standard_normal((S, nq, d)); V = g.standard_normal((S, nkv, d))
    # one visible key: output is that value exactly
    out = orc.attention(q[:1], [0], g.standard_normal((1, nkv, d)), V[:1], real)
    for h in range(nq):
        assert np.array_equal(out[0, h], V[0, h // 2].astype(out.dtype))
    # identical keys: uniform weights, output is the running mean of the values
    K = np.tile(g.standard_normal((1, nkv, d)), (S, 1, 1))
    out = orc.attention(q, np.arange(S), K, V, real)
    run = np.cumsum(V, axis=0) / np.arange(1, S + 1)[:, None, None]
    for h in range(nq):
        assert np.allclose(out[:, h], run[:, h // 2], atol=1e-5)
    # grouped-query attention equals multi-head attention with repeated KV heads
    K = g.standard_normal((S, nkv, d))
    a = orc.attention(q, np.arange(S), K, V, real)
    b = orc.attention(q, np.arange(S), np.repeat(K, 2, axis=1), np.repeat(V, 2, axis=1), real)
    assert np.array_equal(a, b)


# ------------------------------------------------------------------ SwiGLU
@pytest.mark.parametrize("real", REALS)
def test_swiglu_identities(real):
    c = GOLD["silu_values"]
    z = np.array(c["z"])
    assert np.allclose(orc.swiglu(z, np.ones_like(z), real), c["silu"], atol=1e-6)
    g = rng(8)
    z = g.standard_normal(64) * 4; u = g.standard_normal(64)
    s = orc.swiglu(z, np.ones(64), real).astype(np.float64)
    sm = orc.swiglu(-z, np.ones(64), real).astype(np.float64)
    assert np.allclose(sm, s - z, atol=1e-5)              # silu(-z) = silu(z) - z
    assert np.allclose(orc.swiglu(z, u, real), s * u, atol=1e-5)   # the gate multiplies `up`
    big = orc.swiglu(np.array([40.0, -40.0]), np.ones(2), real)
    assert np.allclose(big, [40.0, 0.0], atol=1e-6)


# ------------------------------------------------------------------ whole block
SMALL = synth.BlockShape(hidden=48, n_q_heads=6, n_kv_heads=2, head_dim=8, ffn_dim=80, dtype="f32")


def small_weights(seed, sigma=0.15, shape=SMALL):
    return synth.layer_weights(shape, 0, seed, sigma=sigma)


def block_f64(shape, w, x):
    """Independent float64 evaluation of a whole block on one request in matrix
    form (library matmuls, explicit mask): the special case 'prefill of one
    request' written as a textbook transformer layer."""
    x = x.astype(np.float64)
    W = {k: v.astype(np.float64) for k, v in w.items()}
    S, H = x.shape
    d, nq, nkv = shape.head_dim, shape.n_q_heads, shape.n_kv_heads
    def norm(v, g):
        return v / np.sqrt((v * v).mean(-1, keepdims=True) + shape.rms_eps) * g
    def rot(z):
        half = d // 2
        inv = shape.rope_base ** (-np.arange(half) * 2.0 / d)
        ang = np.arange(S)[:, None] * inv[None, :]
        c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
        z1, z2 = z[..., :half], z[..., half:]
        return np.concatenate([z1 * c - z2 * s, z2 * c + z1 * s], axis=-1)
    u = norm(x, W["attn_norm_g"])
    q = rot((u @ W["wq"].T).reshape(S, nq, d))
    k = rot((u @ W["wk"].T).reshape(S, nkv, d))
    v = (u @ W["wv"].T).reshape(S, nkv, d)
    a, _ = attention_mask_matrix_f64(q, np.arange(S), k, v)
    h = x + a.reshape(S, nq * d) @ W["wo"].T
    r = norm(h, W["ffn_norm_g"])
    gate = r @ W["w_gate"].T
    m = gate / (1 + np.exp(-gate)) * (r @ W["w_up"].T)
    return h + m @ W["w_down"].T


@pytest.mark.parametrize("real", REALS)
def test_block_matches_matrix_form_float64(real):
    w = small_weights(11)
    x = synth.normal((9, SMALL.hidden), 12)
    Kc, Vc = orc.new_cache(SMALL, 9, real)
    out = orc.layer_forward(SMALL, w, x, 0, Kc, Vc, None, real)
    ref = block_f64(SMALL, w, x)
    assert np.abs(out - ref).max() / np.abs(ref).max() < (3e-6 if real == "f32" else 1e-13)
    # the update the block adds is itself resolved (not hidden behind the residual)
    assert np.abs((out - x) - (ref - x)).max() / np.abs(ref - x).max() < (2e-5 if real == "f32" else 1e-12)


def test_block_zero_projections_is_identity():
    w = small_weights(13)
    for k in w:
        if k.startswith("w"):
            w[k] = np.zeros_like(w[k])
    x = synth.normal((5, SMALL.hidden), 14)
    Kc, Vc = orc.new_cache(SMALL, 5)
    assert np.array_equal(orc.layer_forward(SMALL, w, x, 0, Kc, Vc), x)
    # gate = 0 alone switches the FFN off: the output is the attention residual h
    w2 = small_weights(13)
    w2["w_gate"] = np.zeros_like(w2["w_gate"])
    w3 = dict(w2); w3["w_down"] = np.zeros_like(w2["w_down"])
    Kc, Vc = orc.new_cache(SMALL, 5)
    a = orc.layer_forward(SMALL, w2, x, 0, Kc, Vc)
    Kc, Vc = orc.new_cache(SMALL, 5)
    b = orc.layer_forward(SMALL, w3, x, 0, Kc, Vc)
    assert np.array_equal(a, b) and not np.array_equal(a, x)


def test_causal_prefix_invariance_is_bitwise():
    w = small_weights(15)
    x = synth.normal((12, SMALL.hidden), 16)
    Kc, Vc = orc.new_cache(SMALL, 12)
    full = orc.layer_forward(SMALL, w, x, 0, Kc, Vc)
    for p in (1, 5, 11):
        Kp, Vp = orc.new_cache(SMALL, 12)
        part = orc.layer_forward(SMALL, w, x[:p], 0, Kp, Vp)
        assert np.array_equal(part, full[:p])
    # perturbing token j changes no earlier row
    x2 = x.copy(); x2[7] += 1.0
    Kc, Vc = orc.new_cache(SMALL, 12)
    pert = orc.layer_forward(SMALL, w, x2, 0, Kc, Vc)
    assert np.array_equal(pert[:7], full[:7]) and not np.array_equal(pert[7:], full[7:])


def test_selected_rows_equal_full_rows():
    w = small_weights(17)
    x = synth.normal((10, SMALL.hidden), 18)
    Kc, Vc = orc.new_cache(SMALL, 10)
    full = orc.layer_forward(SMALL, w, x, 0, Kc, Vc)
    K2, V2 = orc.new_cache(SMALL, 10)
    some = orc.layer_forward(SMALL, w, x, 0, K2, V2, rows=[9, 0, 4])
    assert np.array_equal(some, full[[9, 0, 4]])
    assert np.array_equal(Kc, K2) and np.array_equal(Vc, V2)


@pytest.mark.parametrize("real", REALS)
def test_cached_decode_equals_full_recompute(real):
    shape = SMALL
    layers = [synth.layer_weights(shape, l, 19, sigma=0.15) for l in range(2)]
    S, steps = 6, 16
    x = synth.normal((S + steps, shape.hidden), 20)
    st = orc.Stage(shape, layers, 1, S + steps, real)
    st.prefill(x[:S], [S])
    for i in range(steps):
        dec = st.decode_step(x[S + i: S + i + 1])
        ref = orc.Stage(shape, layers, 1, S + steps, real).prefill(x[: S + i + 1], [S + i + 1])
        err = np.abs(dec[0] - ref[-1]).max() / np.abs(ref[-1]).max()
        assert err < 1e-6, (i, err)


def test_stage_composition_and_batching():
    shape = SMALL
    layers = [synth.layer_weights(shape, l, 21, sigma=0.15) for l in range(4)]
    lens = [5, 1, 9]
    x = synth.normal((sum(lens), shape.hidden), 22)
    whole = orc.Stage(shape, layers, 3, 12).prefill(x, lens)
    # stage [0,4) == stage [0,2) then stage [2,4)   (Eq. 1 / Eq. 6)
    a = orc.Stage(shape, layers[:2], 3, 12).prefill(x, lens)
    b = orc.Stage(shape, layers[2:], 3, 12).prefill(a, lens)
    assert np.array_equal(whole, b)
    # ragged packed batch == each request alone
    row = 0
    for L in lens:
        alone = orc.Stage(shape, layers, 1, 12).prefill(x[row: row + L], [L])
        assert np.array_equal(alone, whole[row: row + L])
        row += L
    # permuting the requests permutes the output blocks
    perm_x = np.concatenate([x[6:15], x[0:5], x[5:6]])
    perm = orc.Stage(shape, layers, 3, 12).prefill(perm_x, [9, 5, 1])
    assert np.array_equal(perm, np.concatenate([whole[6:15], whole[0:5], whole[5:6]]))
    # batched decode == per-request decode
    st = orc.Stage(shape, layers, 3, 12); st.prefill(x, lens)
    xd = synth.normal((3, shape.hidden), 23)
    both = st.decode_step(xd)
    s1 = orc.Stage(shape, layers, 1, 12); s1.prefill(x[5:6], [1])
    assert np.array_equal(s1.decode_step(xd[1:2])[0], both[1])


def test_float32_oracle_rounding_is_far_below_tolerance():
    wl = synth.WORKLOADS["c1_tiny_f32"]
    w = [synth.layer_weights(wl.shape, 0, wl.seed)]
    x = synth.hidden_states(64, wl.shape, wl.seed + 1)
    a = orc.Stage(wl.shape, w, 1, 80, "f32").prefill(x, [64])
    b = orc.Stage(wl.shape, w, 1, 80, "f64").prefill(x, [64])
    assert np.abs(a - b).max() / np.abs(b).max() < 1e-5
    assert np.abs((a - x) - (b - x)).max() / np.abs(b - x).max() < 1e-5


def test_parameter_count_matches_table1():
    c = GOLD["phi3_medium_params"]
    assert synth.PHI3_MEDIUM.params_per_layer() == c["per_block"]
    total = c["blocks"] * synth.PHI3_MEDIUM.params_per_layer()
    assert total == c["total_blocks"]
    assert 13.0e9 < total < 14.0e9   # "14B" once embeddings are added
