"""Shared plumbing for the GPU parity tests: numpy <-> device tensors, stage
construction on both sides, error metrics.  No decoder-block arithmetic here."""
from __future__ import annotations

import numpy as np

from workloads import synth


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max |ref|  (scale-relative; elementwise ratios blow up at
    the zero crossings of Gaussian data)."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def to_dev(a: np.ndarray, dtype: str):
    import torch
    if dtype == "bf16":
        bits = synth.bf16_bits(a)
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_host(t) -> np.ndarray:
    import torch
    return t.detach().to(torch.float32).cpu().numpy()


def make_config(shape: synth.BlockShape, max_batch: int, max_seq: int, max_prefill: int, flags: int = 0):
    import paper_2511_14450_amd as hyp
    return hyp.stage_config(shape, max_batch, max_seq, max_prefill, flags)


def make_gpu_stage(shape, layers_np, max_batch, max_seq, max_prefill, l_start=0, flags=0):
    import paper_2511_14450_amd as hyp
    cfg = make_config(shape, max_batch, max_seq, max_prefill, flags)
    dev_layers = [{k: to_dev(v, shape.dtype) for k, v in w.items()} for w in layers_np]
    return hyp.stage_create(cfg, l_start, l_start + len(layers_np), dev_layers)
