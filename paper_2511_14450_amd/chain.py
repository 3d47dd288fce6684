"""Stages chained on one device: the model of Eq. 1 cut into T sub-models (Eq. 6),
each a stage of this library, run one after the other the way the tiers of the
pipeline forward activations to each other (Sec. III-B: "batch x sequence x
hidden" values cross every boundary).

`StageChain` only creates the stages and passes buffers along; every decoder
block runs inside the HIP library.  Run as a program it times one request of the
shape the paper evaluates (64 prompt tokens, 128 or 256 generated ones, Sec. V-A)
through all N blocks, with a harness-side embedding table, final RMS Norm and
vocabulary projection in PyTorch closing the greedy loop - those three are not
decoder blocks and stay outside the library.

    python -m paper_2511_14450_amd.chain --model phi3_medium --split 20,13,7 --generate 128
"""
from __future__ import annotations

import argparse
import json
import time
from typing import Callable, Dict, List, Optional, Sequence

import torch

from . import binding


class StageChain:
    """Stages over blocks [b_0, b_1), [b_1, b_2), ... of one model on one device.

    boundaries   [0, p_1, ..., p_{T-1}, N] (0-based block indices; the paper's 1-based
                 partition vector p of Eq. 6 with p_0 = 0 and p_T = N)
    layer_fn(l)  -> dict of device tensors for block l (names of hyp_layer_weights_t);
                 called once per block, the result is dropped after the stage has
                 repacked it
    """

    def __init__(self, shape, boundaries: Sequence[int], layer_fn: Callable[[int], Dict[str, torch.Tensor]],
                 max_batch: int, max_seq: int, max_prefill_tokens: int, flags: int = 0,
                 stream: Optional[torch.cuda.Stream] = None):
        b = [int(v) for v in boundaries]
        if len(b) < 2 or b[0] != 0 or any(b[i] >= b[i + 1] for i in range(len(b) - 1)):
            raise ValueError(f"boundaries must start at 0 and increase strictly: {b}")
        self.shape, self.boundaries = shape, b
        self.stages: List[binding.Stage] = []
        for lo, hi in zip(b[:-1], b[1:]):
            cfg = binding.stage_config(shape, max_batch, max_seq, max_prefill_tokens, flags)
            layers = [layer_fn(l) for l in range(lo, hi)]
            self.stages.append(binding.stage_create(cfg, lo, hi, layers, stream=stream))
            del layers
        self._decode_buf: Dict[int, List[torch.Tensor]] = {}

    @property
    def n_blocks(self) -> int:
        return self.boundaries[-1]

    def prefill(self, hidden: torch.Tensor, seq_lens: Sequence[int]) -> torch.Tensor:
        for st in self.stages:
            hidden = binding.stage_prefill(st, hidden, seq_lens)
        return hidden

    def decode_step(self, hidden: torch.Tensor) -> torch.Tensor:
        """One token per request through every stage; the buffers between stages are
        kept, so a generation loop allocates nothing."""
        rows = hidden.shape[0]
        bufs = self._decode_buf.get(rows)
        if bufs is None or bufs[0].dtype != hidden.dtype:
            bufs = [torch.empty_like(hidden) for _ in self.stages]
            self._decode_buf[rows] = bufs
        for st, out in zip(self.stages, bufs):
            hidden = binding.stage_decode_step(st, hidden, out)
        return hidden

    def context_len(self, request: int) -> int:
        return self.stages[0].context_len(request)

    def destroy(self) -> None:
        for st in self.stages:
            st.destroy()
        self.stages = []


# ----------------------------------------------------------------- whole-model run
MODELS = {
    # blocks, hidden, q heads, kv heads, head dim, ffn dim, vocabulary.  Blocks and hidden
    # size are Table I's; the paper does not list head counts or FFN widths: those are
    # the published ones of the two architectures.
    "phi3_medium": dict(blocks=40, hidden=5120, n_q_heads=40, n_kv_heads=10, head_dim=128, ffn_dim=17920, vocab=32064),
    "llama3_8b": dict(blocks=32, hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn_dim=14336, vocab=128256),
}


class _Shape:
    def __init__(self, m):
        self.hidden, self.n_q_heads, self.n_kv_heads = m["hidden"], m["n_q_heads"], m["n_kv_heads"]
        self.head_dim, self.ffn_dim = m["head_dim"], m["ffn_dim"]
        self.rms_eps, self.rope_base, self.dtype = 1e-5, 10000.0, "bf16"

    def weight_shapes(self):
        H, qd, kvd, I = self.hidden, self.n_q_heads * self.head_dim, self.n_kv_heads * self.head_dim, self.ffn_dim
        return {"attn_norm_g": (H,), "wq": (qd, H), "wk": (kvd, H), "wv": (kvd, H), "wo": (H, qd),
                "ffn_norm_g": (H,), "w_gate": (I, H), "w_up": (I, H), "w_down": (H, I)}


def _synthetic_layer(shape, seed):
    """Seeded N(0, 0.02^2) matrices and 1 + N(0, 0.02^2) gains drawn on the device."""
    gen = torch.Generator(device="cuda")

    def make(l):
        w = {}
        for t, (name, shp) in enumerate(shape.weight_shapes().items()):
            gen.manual_seed(seed * 1000 + (l + 1) * 16 + t)
            z = torch.randn(shp, generator=gen, device="cuda", dtype=torch.float32) * 0.02
            if name.endswith("_g"):
                z += 1.0
            w[name] = z.to(torch.bfloat16).contiguous()
        return w
    return make


def run_whole_model(model: str, split: Sequence[int], prompt: int, generate: int, batch: int = 1,
                    seed: int = 251114450, repeats: int = 3) -> dict:
    """Greedy generation of `generate` tokens after a `prompt`-token prefill through all
    blocks of `model`, cut into len(split) stages of split[j] blocks.  Returns timings."""
    m = MODELS[model]
    if sum(split) != m["blocks"]:
        raise ValueError(f"split {list(split)} does not add up to the {m['blocks']} blocks of {model}")
    shape = _Shape(m)
    bounds = [0]
    for n in split:
        bounds.append(bounds[-1] + int(n))
    n_probe = 16  # decode steps per stage and repetition of the per-stage timing below
    chain = StageChain(shape, bounds, _synthetic_layer(shape, seed), batch, prompt + generate + 2 * n_probe, batch * prompt)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed + 5)
    emb = torch.randn((m["vocab"], m["hidden"]), generator=gen, device="cuda").to(torch.bfloat16)
    head = (torch.randn((m["vocab"], m["hidden"]), generator=gen, device="cuda") * 0.02).to(torch.bfloat16)
    tokens0 = torch.randint(0, m["vocab"], (batch * prompt,), generator=gen, device="cuda")
    picked = torch.empty((generate, batch), dtype=torch.long, device="cuda")

    def next_token(h):  # final RMS Norm (unit gain) + vocabulary projection + argmax, harness side
        hf = h.float()
        hn = (hf * torch.rsqrt(hf.pow(2).mean(-1, keepdim=True) + shape.rms_eps)).to(torch.bfloat16)
        return (hn @ head.t()).argmax(-1)

    stage_ms = [0.0] * len(split)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(split) + 1)] for _ in range(2)]

    def one_request(timed_stages: bool):
        h = emb[tokens0]
        lens = [prompt] * batch
        if timed_stages:
            ev[0][0].record()
            for j, st in enumerate(chain.stages):
                h = binding.stage_prefill(st, h, lens)
                ev[0][j + 1].record()
        else:
            h = chain.prefill(h, lens)
        last = h.view(batch, prompt, -1)[:, -1, :]
        tok = next_token(last)
        picked[0] = tok
        for s in range(1, generate):
            h = chain.decode_step(emb[tok])
            tok = next_token(h)
            picked[s] = tok

    one_request(False)  # warm-up: first-use graph capture, allocator
    torch.cuda.synchronize()
    first = picked.clone()
    times = []
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        one_request(False)
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
    if not torch.equal(first, picked):
        raise RuntimeError("generation is not reproducible from run to run")
    # per-stage decode time: what a partitioner needs as f_i / C_j of this device
    h = emb[picked[-1]]
    outs = [torch.empty_like(h) for _ in chain.stages]
    for rep in range(2):
        for j, st in enumerate(chain.stages):
            ev[1][0].record()
            for _ in range(n_probe):
                binding.stage_decode_step(st, h, outs[j])
            ev[1][1].record()
            torch.cuda.synchronize()
            stage_ms[j] = ev[1][0].elapsed_time(ev[1][1]) / n_probe
    one_request(True)
    torch.cuda.synchronize()
    prefill_ms = [ev[0][j].elapsed_time(ev[0][j + 1]) for j in range(len(split))]
    e2e = sorted(times)[len(times) // 2]
    res = {"workload": "whole-model chain, one request at a time", "model": model, "split": [int(v) for v in split],
           "batch": batch, "prompt_tokens": prompt, "generated_tokens": generate, "dtype": "bf16", "data": "synthetic",
           "end_to_end_s": e2e, "s_per_generated_token": e2e / generate,
           "stage_prefill_ms": prefill_ms, "stage_decode_ms_per_token": stage_ms,
           "tokens_head": [int(v) for v in picked[:8, 0].tolist()]}
    chain.destroy()
    return res


def _model_spec(model):
    """A name from MODELS, or a dict with the same keys (blocks, hidden, n_q_heads, n_kv_heads,
    head_dim, ffn_dim) for any other bf16 model."""
    return MODELS[model] if isinstance(model, str) else dict(model)


def measure_block_costs(model, prompt: int, generate: int, batch: int = 1, seed: int = 251114450):
    """What Algorithm 1 needs to know about a block, measured on this device: f = the
    seconds one block spends on a request of the given shape (prefill + every decode
    step; all blocks of a model have one shape, so one block is measured), m = the bytes
    a block adds to a stage (repacked weights + its share of the KV cache)."""
    m = _model_spec(model)
    shape = _Shape(m)
    chain = StageChain(shape, [0, 1], _synthetic_layer(shape, seed), batch, prompt + generate + 1, batch * prompt)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed + 6)
    x = torch.randn((batch * prompt, m["hidden"]), generator=gen, device="cuda").to(torch.bfloat16)
    xd = torch.randn((batch, m["hidden"]), generator=gen, device="cuda").to(torch.bfloat16)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    seconds = 0.0
    for rep in range(2):  # the first pass warms up (graph capture)
        e0.record()
        chain.prefill(x, [prompt] * batch)
        for _ in range(generate - 1):
            chain.decode_step(xd)
        e1.record()
        torch.cuda.synchronize()
        seconds = e0.elapsed_time(e1) * 1e-3
    cfg = binding.stage_config(shape, batch, prompt + generate + 1, batch * prompt)
    bytes_per_block = binding.stage_workspace_bytes(cfg, 0, 2) - binding.stage_workspace_bytes(cfg, 0, 1)
    chain.destroy()
    return seconds, float(bytes_per_block)


def plan_split(model, tiers: Sequence[Sequence[float]], prompt: int, generate: int, eps: float, batch: int = 1):
    """HypSplit-DP (Sec. IV-A) on measured block costs.  tiers = [(capacity, memory GB), ...]
    in the order the pipeline visits them; capacities are relative (Table I lists TOPS):
    the largest stands for this device, f_i / C_j is then the time of block i on tier j."""
    n = _model_spec(model)["blocks"]
    f1, m1 = measure_block_costs(model, prompt, generate, batch)
    cap_ref = max(float(c) for c, _ in tiers)
    C = [float(c) / cap_ref for c, _ in tiers]
    M = [float(g) * 1e9 for _, g in tiers]
    t0 = time.perf_counter()
    p, tau = binding.hypsplit_dp([f1] * n, [m1] * n, C, M, eps)
    dt = time.perf_counter() - t0
    plan = {"model": model if isinstance(model, str) else "custom", "blocks": n, "tiers": [[float(c), float(g)] for c, g in tiers], "eps": eps,
            "f_seconds_per_block": f1, "m_bytes_per_block": m1, "p": p, "tau_seconds": tau,
            "hypsplit_dp_seconds": dt}
    if p is not None:
        b = [0] + p + [n]
        plan["blocks_per_tier"] = [b[j + 1] - b[j] for j in range(len(tiers))]
        plan["tier_load_seconds"] = [f1 * (b[j + 1] - b[j]) / C[j] for j in range(len(tiers))]
    return plan


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--model", choices=sorted(MODELS), default="phi3_medium")
    ap.add_argument("--split", default=None, help="blocks per stage, e.g. 20,13,7 (default: four equal stages)")
    ap.add_argument("--tiers", default=None,
                    help="plan the split with HypSplit-DP instead: capacity:memoryGB per tier, e.g. 67:8,157:16,200:32")
    ap.add_argument("--eps", type=float, default=1e-3, help="precision of the binary search (Sec. V-A uses 1e-3)")
    ap.add_argument("--prompt", type=int, default=64)
    ap.add_argument("--generate", type=int, default=128)
    ap.add_argument("--batch", type=int, default=1)
    a = ap.parse_args()
    n = MODELS[a.model]["blocks"]
    if a.tiers:
        tiers = [tuple(float(v) for v in t.split(":")) for t in a.tiers.split(",")]
        plan = plan_split(a.model, tiers, a.prompt, a.generate, a.eps, a.batch)
        print(json.dumps(plan))
        if plan["p"] is None:
            raise SystemExit("no partition fits the tiers' memory")
        split = plan["blocks_per_tier"]
    else:
        split = [int(v) for v in a.split.split(",")] if a.split else [n // 4] * 4
    print(json.dumps(run_whole_model(a.model, split, a.prompt, a.generate, a.batch)))


if __name__ == "__main__":
    main()
