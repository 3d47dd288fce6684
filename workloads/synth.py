"""Seeded synthetic inputs for a pipeline stage of decoder blocks.

This module only *draws numbers and rounds them*: it holds none of the
decoder-block arithmetic.  Both the CPU oracle's tests and the HIP library's
tests/bench import it so that the two sides see the very same bytes.

Recipe (stands in for real Phi-3-medium weights and prompts, which the paper
ran (Table I, Sec. V-A) but which are neither available nor needed here):
  * projection matrices  ~ N(0, 0.02^2), row-major [out, in]
  * RMSNorm gains        = 1 + N(0, 0.02^2)   (so a dropped gain is visible)
  * hidden states        ~ N(0, 1)
  * bf16 workloads round every tensor once to bf16 (round-to-nearest-even);
    the oracle receives those rounded values widened to float32, the GPU path
    receives the 16-bit patterns.
  * ragged context lengths ~ U{lo..hi}

Every tensor is drawn in fixed-size chunks, each from its own Philox stream
keyed by (seed, tensor tag, chunk index), so the values do not depend on the
number of worker threads.
"""
from __future__ import annotations

import concurrent.futures as _cf
import dataclasses
import os
from typing import Dict, List, Sequence

import numpy as np

BASE_SEED = 251114450
_CHUNK = 1 << 22  # elements per Philox stream

WEIGHT_NAMES = (
    "attn_norm_g", "wq", "wk", "wv", "wo", "ffn_norm_g", "w_gate", "w_up", "w_down",
)


@dataclasses.dataclass(frozen=True)
class BlockShape:
    """Shape of one decoder block (Table I gives depth and hidden size only;
    head counts, FFN width, eps and RoPE base come from the workload list)."""
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_dim: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    dtype: str = "bf16"  # "f32" | "bf16"

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def weight_shapes(self) -> Dict[str, tuple]:
        H, I = self.hidden, self.ffn_dim
        return {
            "attn_norm_g": (H,),
            "wq": (self.q_dim, H),
            "wk": (self.kv_dim, H),
            "wv": (self.kv_dim, H),
            "wo": (H, self.q_dim),
            "ffn_norm_g": (H,),
            "w_gate": (I, H),
            "w_up": (I, H),
            "w_down": (H, I),
        }

    def params_per_layer(self) -> int:
        return sum(int(np.prod(s)) for n, s in self.weight_shapes().items() if n.startswith("w"))


TINY = BlockShape(256, 4, 2, 64, 1024, dtype="f32")
TINY_BF16 = dataclasses.replace(TINY, dtype="bf16")
PHI3_MEDIUM = BlockShape(5120, 40, 10, 128, 17920, dtype="bf16")
# the paper's second model (Table I: 32 blocks, hidden 4096, GQA); head counts and FFN width are
# the architecture's published ones, the paper does not list them
LLAMA3_8B = BlockShape(4096, 32, 8, 128, 14336, dtype="bf16")


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int
    shape: BlockShape
    n_layers: int
    prefill_lens: tuple          # prompt length of every request
    decode_steps: int
    ragged_ctx: tuple = ()       # (lo, hi): context lengths drawn uniformly; overrides prefill_lens

    @property
    def seed(self) -> int:
        return BASE_SEED + 1000 * self.index

    @property
    def batch(self) -> int:
        return len(self.lengths())

    def lengths(self) -> List[int]:
        if self.ragged_ctx:
            lo, hi = self.ragged_ctx
            return ragged_lengths(len(self.prefill_lens), lo, hi, self.seed + 7)
        return list(self.prefill_lens)


WORKLOADS = {
    "c1_tiny_f32": Workload("c1_tiny_f32", 0, TINY, 1, (64,), 16),
    "c2_layer_prefill": Workload("c2_layer_prefill", 1, PHI3_MEDIUM, 1, (512,) * 4, 0),
    "c3_stage10": Workload("c3_stage10", 2, PHI3_MEDIUM, 10, (2048,) * 8, 128),
    "c4_decode_heavy": Workload("c4_decode_heavy", 3, PHI3_MEDIUM, 10, (0,) * 32, 256, (1024, 4096)),
    "c5_long": Workload("c5_long", 4, PHI3_MEDIUM, 20, (8192,) * 8, 1024),
    "n4_llama3_stage8": Workload("n4_llama3_stage8", 5, LLAMA3_8B, 8, (2048,) * 8, 128),
}


# ----------------------------------------------------------------------------
# bf16 helpers (bit manipulation only)
# ----------------------------------------------------------------------------
def bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> uint16 bf16 patterns, round-to-nearest-even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_widen(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 patterns -> float32 with the same value."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def round_bf16(a: np.ndarray) -> np.ndarray:
    return bf16_widen(bf16_bits(a))


# ----------------------------------------------------------------------------
# chunked, thread-count independent normal draws
# ----------------------------------------------------------------------------
def _draw_chunk(seed: int, tag: int, chunk: int, n: int) -> np.ndarray:
    gen = np.random.Generator(np.random.Philox(key=[(seed << 20) ^ tag, chunk]))
    return gen.standard_normal(n, dtype=np.float32)


def normal(shape: Sequence[int], seed: int, tag: int = 0, workers: int | None = None) -> np.ndarray:
    """Standard normal float32 tensor, reproducible from (seed, tag, shape)."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    n_chunks = (n + _CHUNK - 1) // _CHUNK
    if workers is None:
        workers = min(16, os.cpu_count() or 1)

    def work(c):
        lo = c * _CHUNK
        hi = min(n, lo + _CHUNK)
        out[lo:hi] = _draw_chunk(seed, tag, c, hi - lo)

    if n_chunks <= 1 or workers <= 1:
        for c in range(n_chunks):
            work(c)
    else:
        with _cf.ThreadPoolExecutor(workers) as ex:
            list(ex.map(work, range(n_chunks)))
    return out.reshape(tuple(shape))


def _finish(a: np.ndarray, dtype: str) -> np.ndarray:
    return round_bf16(a) if dtype == "bf16" else a


def layer_weights(shape: BlockShape, layer: int, seed: int, sigma: float = 0.02) -> Dict[str, np.ndarray]:
    """float32 arrays (already bf16-representable when shape.dtype == 'bf16')."""
    out = {}
    for t, (name, shp) in enumerate(shape.weight_shapes().items()):
        z = normal(shp, seed, tag=(layer + 1) * 16 + t)
        z *= np.float32(sigma)
        if name.endswith("_g"):
            z += np.float32(1.0)
        out[name] = _finish(z, shape.dtype)
    return out


def hidden_states(n_rows: int, shape: BlockShape, seed: int) -> np.ndarray:
    return _finish(normal((n_rows, shape.hidden), seed, tag=0), shape.dtype)


def ragged_lengths(batch: int, lo: int, hi: int, seed: int) -> List[int]:
    gen = np.random.Generator(np.random.Philox(key=[seed, 0]))
    return [int(v) for v in gen.integers(lo, hi + 1, size=batch)]


def readout_tables(shape: BlockShape, vocab: int, seed: int):
    """Harness-only tables for the greedy-token check: a stage has no logits, so
    the tests project its last hidden row on E [vocab, hidden] ~ N(0, 0.02^2)
    and feed row argmax of Emb [vocab, hidden] ~ N(0, 1) back in."""
    E = _finish(normal((vocab, shape.hidden), seed, tag=9001) * np.float32(0.02), shape.dtype)
    Emb = _finish(normal((vocab, shape.hidden), seed, tag=9002), shape.dtype)
    return E, Emb
