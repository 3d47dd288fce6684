"""ctypes binding of the C oracle (test infrastructure only).

Every function takes and returns numpy arrays; `real` selects the float32 build
(the precision the oracle is specified in) or the float64 build (used to bound
the oracle's own rounding).  See hyp_oracle.c for what each routine computes and
which passage of the paper it follows.
"""
from __future__ import annotations

import ctypes as C
from typing import Dict, List, Optional, Sequence

import numpy as np

from . import build as _build

_LIBS: Dict[str, C.CDLL] = {}
_NP = {"f32": np.float32, "f64": np.float64}


class _Shape(C.Structure):
    _fields_ = [("hidden", C.c_int), ("n_q_heads", C.c_int), ("n_kv_heads", C.c_int),
                ("head_dim", C.c_int), ("ffn_dim", C.c_int),
                ("rms_eps", C.c_double), ("rope_base", C.c_double)]


class _Layer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("attn_norm_g", "wq", "wk", "wv", "wo", "ffn_norm_g", "w_gate", "w_up", "w_down")]


def _lib(real: str) -> C.CDLL:
    if real not in _LIBS:
        _build.build()
        lib = C.CDLL(str(_build.lib_path(real)))
        lib.orc_real_bytes.restype = C.c_int
        assert lib.orc_real_bytes() == np.dtype(_NP[real]).itemsize
        _LIBS[real] = lib
    return _LIBS[real]


def _arr(a, real) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=_NP[real])


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _ints(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _shape(s) -> _Shape:
    return _Shape(s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn_dim,
                  float(s.rms_eps), float(s.rope_base))


def rmsnorm(x, g, eps, real="f32"):
    x = _arr(x, real); g = _arr(g, real)
    T, H = x.shape
    y = np.empty_like(x)
    _lib(real).orc_rmsnorm(_p(x), _p(g), C.c_double(eps), T, H, _p(y))
    return y


def linear(x, W, real="f32"):
    x = _arr(x, real); W = _arr(W, real)
    T, K = x.shape
    N, K2 = W.shape
    assert K == K2
    y = np.empty((T, N), dtype=_NP[real])
    _lib(real).orc_linear(_p(x), _p(W), T, K, N, _p(y))
    return y


def rope(z, pos, base=10000.0, real="f32"):
    """z [T, heads, d] -> rotated copy."""
    z = _arr(z, real).copy(); pos = _ints(pos)
    T, nh, d = z.shape
    assert pos.shape == (T,)
    _lib(real).orc_rope(_p(z), _p(pos), T, nh, d, C.c_double(base))
    return z


def softmax(s, real="f32"):
    s = _arr(s, real).copy()
    assert s.ndim == 1
    _lib(real).orc_softmax(_p(s), s.shape[0])
    return s


def attention(q, q_pos, K, V, real="f32", return_probs=False):
    """q [R, n_q, d], K/V [n_keys, n_kv, d] -> out [R, n_q, d] (and probs [n_q, R, n_keys])."""
    q = _arr(q, real); K = _arr(K, real); V = _arr(V, real); q_pos = _ints(q_pos)
    R, nq, d = q.shape
    nk, nkv, d2 = K.shape
    assert d == d2 and V.shape == K.shape and nq % nkv == 0
    assert q_pos.shape == (R,) and (R == 0 or (q_pos.max() < nk and q_pos.min() >= 0))
    out = np.empty_like(q)
    probs = np.empty((nq, R, nk), dtype=_NP[real]) if return_probs else None
    _lib(real).orc_attention(_p(q), _p(q_pos), R, _p(K), _p(V), nk, nq, nkv, d, _p(out), _p(probs))
    return (out, probs) if return_probs else out


def swiglu(gate, up, real="f32"):
    gate = _arr(gate, real); up = _arr(up, real)
    m = np.empty_like(gate)
    _lib(real).orc_swiglu(_p(gate), _p(up), C.c_size_t(gate.size), _p(m))
    return m


def _layer_struct(w: dict, real: str, keep: list) -> _Layer:
    L = _Layer()
    for name, _ in _Layer._fields_:
        a = _arr(w[name], real)
        keep.append(a)
        setattr(L, name, a.ctypes.data)
    return L


def new_cache(shape, cap: int, real="f32"):
    kvd = shape.n_kv_heads * shape.head_dim
    return (np.zeros((cap, kvd), dtype=_NP[real]), np.zeros((cap, kvd), dtype=_NP[real]))


def layer_forward(shape, w: dict, x, pos0: int, Kc, Vc, rows: Optional[Sequence[int]] = None, real="f32"):
    """One block over the S rows of x for one request; Kc/Vc [cap, n_kv*d] updated in place."""
    x = _arr(x, real)
    S, H = x.shape
    assert H == shape.hidden and Kc.dtype == _NP[real] and Kc.flags.c_contiguous
    assert pos0 + S <= Kc.shape[0]
    keep: list = []
    L = _layer_struct(w, real, keep)
    sh = _shape(shape)
    if rows is None:
        r, n = None, 0
        out = np.empty((S, H), dtype=_NP[real])
    else:
        r = _ints(rows); n = len(r)
        assert n == 0 or (r.min() >= 0 and r.max() < S)
        out = np.empty((n, H), dtype=_NP[real])
    _lib(real).orc_layer_forward(C.byref(sh), C.byref(L), _p(x), S, pos0, _p(Kc), _p(Vc),
                                 _p(r), n, _p(out))
    return out


class Stage:
    """Stage state for the oracle: the weights of blocks [l_start, l_end) and a plain
    cache slab [n_layers][batch][cap][n_kv*d]."""

    def __init__(self, shape, layers: List[dict], batch: int, cap: int, real="f32"):
        self.shape, self.real, self.batch, self.cap = shape, real, batch, cap
        self._keep: list = []
        self._layers = (_Layer * len(layers))(*[_layer_struct(w, real, self._keep) for w in layers])
        self.n_layers = len(layers)
        kvd = shape.n_kv_heads * shape.head_dim
        self.K = np.zeros((self.n_layers, batch, cap, kvd), dtype=_NP[real])
        self.V = np.zeros_like(self.K)
        self.lens = np.zeros(batch, dtype=np.int32)

    def _run(self, x, seq_lens, pos0):
        x = _arr(x, self.real)
        out = np.empty_like(x)
        sh = _shape(self.shape)
        seq_lens = _ints(seq_lens); pos0 = _ints(pos0)
        assert x.shape[0] == int(seq_lens.sum())
        assert int((seq_lens + pos0).max()) <= self.cap
        _lib(self.real).orc_stage_forward(C.byref(sh), self._layers, self.n_layers, _p(x), _p(seq_lens),
                                          _p(pos0), len(seq_lens), _p(self.K), _p(self.V), self.cap, _p(out))
        return out

    def prefill(self, x, seq_lens):
        assert len(seq_lens) == self.batch
        out = self._run(x, seq_lens, np.zeros(self.batch, dtype=np.int32))
        self.lens = _ints(seq_lens).copy()
        return out

    def decode_step(self, x):
        out = self._run(x, np.ones(self.batch, dtype=np.int32), self.lens)
        self.lens = self.lens + 1
        return out
