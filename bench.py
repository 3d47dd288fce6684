#!/usr/bin/env python3
"""Throughput of one pipeline stage on one MI355X.

A *step* is one pass of the whole stage hot path over one synthetic batch:
stage_prefill over the prompts, then the workload's KV-cached stage_decode_step
calls.  Default workload: c5_long = 20 Phi-3-medium-shaped blocks (half of the 40
of Table I), prefill 8 x 8192, then 1024 decode steps at batch 8 - the largest
configuration that fits one GPU.

Prints ONE JSON line: whole-step tokens/s (prefill and decode tokens together,
with the two phases also given separately), the roofline of the kernel class
that takes the most time (durations from HIP events recorded by the library
around every launch of that class), the other configurations in brief, and the
CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from workloads import synth  # noqa: E402

PEAK_BF16_TFLOPS = 2516.6   # MI355X dense bf16 MFMA: 256 CU x 4096 FLOP/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
DEFAULT_WORKLOAD = "c5_long"
KERNEL_TIMING = ("HIP events recorded by the library on the stage's stream around every launch of a class, in one extra "
                 "pass with graph replay off: a duration includes the gap to the next event (2-3 us more than the "
                 "kernel's own time in a rocprofv3 trace)")


def progress(msg):
    """One line on stderr per finished part (the JSON line on stdout stays alone)."""
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def traffic_file(workload):
    return os.path.join(ROOT, "profiles", f"traffic_{workload}.json")


def kernel_sources_digest():
    """sha256 over the HIP sources: traffic counters are only quoted for the kernels they were taken from."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2511_14450_amd", "csrc")
    for name in sorted(os.listdir(d)):
        with open(os.path.join(d, name), "rb") as f:
            h.update(name.encode()); h.update(f.read())
    return h.hexdigest()


def committed_traffic(workload):
    """{kernel class: HBM bytes per launch} from the committed rocprofv3 --pmc summary, or {} when there
    is none for this workload or it belongs to older kernel sources."""
    try:
        with open(traffic_file(workload)) as f:
            t = json.load(f)
    except OSError:
        return {}
    if t.get("workload") != workload or t.get("sources_sha256") != kernel_sources_digest():
        return {}
    return t.get("hbm_bytes_per_launch", {})


def device_weights(shape, n_layers, seed):
    """Seeded N(0, 0.02^2) matrices and 1 + N(0, 0.02^2) gains, drawn on the device
    (10-20 layers of 341 M parameters each are too slow to draw on the host)."""
    import torch
    gen = torch.Generator(device="cuda")
    layers = []
    for l in range(n_layers):
        w = {}
        for t, (name, shp) in enumerate(shape.weight_shapes().items()):
            gen.manual_seed(seed * 1000 + (l + 1) * 16 + t)
            z = torch.randn(shp, generator=gen, device="cuda", dtype=torch.float32) * 0.02
            if name.endswith("_g"):
                z += 1.0
            w[name] = z.to(torch.bfloat16).contiguous()
        layers.append(w)
    return layers


def device_normal(shape, seed):
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    return torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16).contiguous()


def cpu_baseline(wl, prompt=2048, decode=32):
    """The oracle as it stands on a bounded sample: ONE block of the workload's
    shape over one request of `prompt` tokens plus `decode` cached steps.  Its
    tokens/s is divided by the stage's block count to be comparable with `value`."""
    from oracle import hyp_oracle as orc
    shape = wl.shape
    w = synth.layer_weights(shape, 0, wl.seed)
    x = synth.hidden_states(prompt + decode, shape, wl.seed + 1)
    st = orc.Stage(shape, [w], 1, prompt + decode, "f32")
    t0 = time.perf_counter()
    st.prefill(x[:prompt], [prompt])
    for i in range(decode):
        st.decode_step(x[prompt + i: prompt + i + 1])
    dt = time.perf_counter() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {
        "value": (prompt + decode) / dt / wl.n_layers,
        "unit": "tokens/s",
        "cores": cores,
        "kind": "oracle",
        "seconds": dt,
        "sample": f"1 of {wl.n_layers} blocks of {wl.name}, 1 request: {prompt} prompt tokens + {decode} cached decode steps "
                  f"(the workload's requests have {max(wl.lengths())} prompt tokens, whose longer attention the sample does "
                  f"not pay); tokens/s divided by {wl.n_layers} blocks",
    }


def run_workload(wl, steps, warmup, no_graph=False, traffic_calibration=False, profile_stride=16, paged=False):
    """Time `steps` steps of one workload (after `warmup` untimed ones), then one more pass with events
    around the launches of every kernel class (all prefill launches; every `profile_stride`-th decode step)."""
    import torch
    import paper_2511_14450_amd as hyp
    from paper_2511_14450_amd import binding
    shape = wl.shape
    lens = wl.lengths()
    B, T = len(lens), sum(lens)
    n_dec = wl.decode_steps
    flags = (binding.HYP_FLAG_NO_GRAPH if no_graph else 0) | (binding.HYP_FLAG_PAGED_KV if paged else 0)
    cfg = hyp.stage_config(shape, B, max(lens) + n_dec, T, flags=flags)
    layers = device_weights(shape, wl.n_layers, wl.seed)
    stage = hyp.stage_create(cfg, 0, wl.n_layers, layers)
    del layers
    if paged:  # the cache's 128-key pages handed to the requests in a seeded shuffled order
        ppr = -(-((max(lens) + n_dec + 63) // 64 * 64) // binding.HYP_KV_PAGE_KEYS)
        perm = np.random.Generator(np.random.Philox(key=[wl.seed, 11])).permutation(B * ppr)
        stage.set_page_table([[int(v) for v in perm[r * ppr:(r + 1) * ppr]] for r in range(B)])
    torch.cuda.empty_cache()
    assert stage.uses_mfma(), "the bench workloads must run on the MFMA path"

    x = device_normal((T, shape.hidden), wl.seed + 1)
    xd = device_normal((max(min(n_dec, 128), 1), B, shape.hidden), wl.seed + 2)  # decode inputs, reused every 128 steps
    y = torch.empty_like(x)
    yd = torch.empty((B, shape.hidden), dtype=torch.bfloat16, device="cuda")

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    pre_ms, dec_ms = [], []

    def step(record):
        if record:
            ev[0].record()
        stage.prefill(x, lens, y)
        if record:
            ev[1].record()
        for s in range(n_dec):
            stage.decode_step(xd[s % xd.shape[0]], yd)
        if record:
            ev[2].record()

    if traffic_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty_like(src)
        dst.copy_(src)      # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    progress(f"{wl.name}: stage created ({wl.n_layers} blocks), {warmup} warm-up + {steps} timed steps")
    for _ in range(warmup):
        step(False)
        torch.cuda.synchronize()
        progress(f"{wl.name}: warm-up step done")
    t0 = time.perf_counter()
    for i in range(steps):
        step(True)
        torch.cuda.synchronize()
        progress(f"{wl.name}: timed step {i + 1} of {steps} done")
        pre_ms.append(ev[0].elapsed_time(ev[1]))
        dec_ms.append(ev[1].elapsed_time(ev[2]))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / steps * 1e3
    tokens_per_step = T + B * n_dec
    pre = float(np.median(pre_ms))
    dec = float(np.median(dec_ms))

    # per-kernel-class durations: one extra pass with events around the launches
    H, I, qd, kvd = shape.hidden, shape.ffn_dim, shape.q_dim, shape.kv_dim
    ctx_mean = float(np.mean(lens)) + (n_dec - 1) / 2.0 + 1
    gemm_flops = {"gemm_qkv": 2.0 * T * (qd + 2 * kvd) * H, "gemm_o": 2.0 * T * H * qd,
                  "gemm_gateup": 2.0 * T * 2 * I * H, "gemm_down": 2.0 * T * H * I,
                  "attn_prefill": sum(2.0 * 2 * shape.n_q_heads * shape.head_dim * L * (L + 1) / 2 for L in lens)}
    gemv_bytes = {"gemv_qkv": 2.0 * (qd + 2 * kvd) * H, "gemv_o": 2.0 * H * qd, "gemv_gateup": 2.0 * 2 * I * H,
                  "gemv_down": 2.0 * H * I, "attn_decode": 2.0 * 2 * kvd * B * ctx_mean}
    acc = {}
    stage.profile(list(gemm_flops))
    stage.prefill(x, lens, y)
    for c in gemm_flops:
        acc[c] = stage.profile_read(c)
    stage.profile([])
    sampled_ctx = []
    for s in range(n_dec):
        if s % profile_stride == 0:
            stage.profile(list(gemv_bytes))
            stage.decode_step(xd[s % xd.shape[0]], yd)
            for c in gemv_bytes:
                ms, n = stage.profile_read(c)
                acc[c] = (acc.get(c, (0.0, 0))[0] + ms, acc.get(c, (0.0, 0))[1] + n)
            stage.profile([])
            sampled_ctx.append(float(np.mean(lens)) + s + 1)
        else:
            stage.decode_step(xd[s % xd.shape[0]], yd)
    torch.cuda.synchronize()
    if sampled_ctx:  # the attention's algorithmic bytes at the contexts of the sampled steps
        gemv_bytes_prof = dict(gemv_bytes, attn_decode=2.0 * 2 * kvd * B * float(np.mean(sampled_ctx)))
    rows = []
    traffic = committed_traffic(wl.name)
    for c, (ms, n) in acc.items():
        if n == 0:
            continue
        avg_s = ms / n * 1e-3
        if c in gemm_flops:
            ach, peak, unit, bound = gemm_flops[c] / avg_s / 1e12, PEAK_BF16_TFLOPS, "TFLOP/s", "mfma"
            total_ms = ms / n * wl.n_layers
        else:
            ach, peak, unit, bound = gemv_bytes_prof[c] / avg_s / 1e9, PEAK_HBM_GBS, "GB/s", "hbm"
            total_ms = ms / n * wl.n_layers * n_dec
        rows.append({"kernel": c, "bound": bound, "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak,
                     "traffic": traffic.get(c), "launches_timed": n, "avg_ms": ms / n, "total_ms_per_step": total_ms})
    rows.sort(key=lambda r: -r["total_ms_per_step"])
    dominant = rows[0]

    out = {
        "value": tokens_per_step / (ms_per_step * 1e-3),
        "ms_per_step": ms_per_step,
        "config": {"workload": wl.name + (" (paged KV cache, shuffled 128-key pages)" if paged else ""), "layers": wl.n_layers, "batch": B, "prefill_tokens": T,
                   "decode_steps": n_dec, "hidden": H, "ffn": I, "q_heads": shape.n_q_heads,
                   "kv_heads": shape.n_kv_heads},
        "prefill_tokens_per_s": T / (pre * 1e-3),
        "decode_tokens_per_s": (B * n_dec / (dec * 1e-3)) if n_dec else None,
        "prefill_ms": pre, "decode_ms_per_step": dec / n_dec if n_dec else None,
        "prefill_gemm_frac_of_mfma_peak": sum(gemm_flops[k] for k in ("gemm_qkv", "gemm_o", "gemm_gateup", "gemm_down"))
        * wl.n_layers / (pre * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "prefill_frac_of_mfma_peak_with_attention": sum(gemm_flops.values()) * wl.n_layers / (pre * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "decode_frac_of_hbm_peak": (wl.n_layers * sum(gemv_bytes.values()) / (dec / n_dec * 1e-3) / 1e9 / PEAK_HBM_GBS)
        if n_dec else None,
        "roofline": {k: dominant[k] for k in ("kernel", "bound", "achieved", "peak", "unit", "frac", "traffic")},
        "kernel_timing": KERNEL_TIMING,
        "kernels": rows,
    }
    stage.destroy()
    del stage, x, y, xd, yd
    torch.cuda.empty_cache()
    progress(f"{wl.name}: per-kernel pass done")
    return out


def brief(r):
    """One other configuration in a few figures."""
    keep = ("prefill_ms", "prefill_tokens_per_s", "prefill_gemm_frac_of_mfma_peak", "decode_ms_per_step",
            "decode_tokens_per_s", "decode_frac_of_hbm_peak")
    out = {"workload": r["config"]["workload"], "layers": r["config"]["layers"], "batch": r["config"]["batch"],
           "prefill_tokens": r["config"]["prefill_tokens"], "decode_steps": r["config"]["decode_steps"],
           "tokens_per_s": r["value"]}
    out.update({k: r[k] for k in keep})
    out["kernel_frac_of_peak"] = {k["kernel"]: round(k["frac"], 4) for k in r["kernels"]}
    return out


def prefill_only_line(name, repeats=20):
    """Tokens/s of a prefill-only configuration (c2: one block, 4 x 512), timed with events."""
    import torch
    import paper_2511_14450_amd as hyp
    wl = synth.WORKLOADS[name]
    lens = wl.lengths()
    T = sum(lens)
    cfg = hyp.stage_config(wl.shape, len(lens), max(lens), T)
    stage = hyp.stage_create(cfg, 0, wl.n_layers, device_weights(wl.shape, wl.n_layers, wl.seed))
    x = device_normal((T, wl.shape.hidden), wl.seed + 1)
    y = torch.empty_like(x)
    for _ in range(3):
        stage.prefill(x, lens, y)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(repeats):
        stage.prefill(x, lens, y)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / repeats
    stage.destroy()
    flops = 2.0 * T * wl.shape.params_per_layer() * wl.n_layers
    return {"workload": name, "layers": wl.n_layers, "batch": len(lens), "prefill_tokens": T, "decode_steps": 0,
            "prefill_ms": ms, "prefill_tokens_per_s": T / (ms * 1e-3),
            "prefill_gemm_frac_of_mfma_peak": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}


def gemm_constant_operands_tflops(wl):
    """TFLOP/s of the gate/up prefill GEMM kernel when every weight and activation is one
    constant: the same instruction stream as in the timed run, but operands that barely
    toggle the datapath, so the chip holds its clock.  The gap to the timed run's figure is
    what the data, not the kernel's schedule, costs."""
    import torch
    import paper_2511_14450_amd as hyp
    shape = wl.shape
    lens = [2048] * 8
    T = sum(lens)
    cfg = hyp.stage_config(shape, len(lens), max(lens), T)
    w = {n: torch.full(shp, 1.0 if n.endswith("_g") else 0.0078125, dtype=torch.bfloat16, device="cuda")
         for n, shp in shape.weight_shapes().items()}
    stage = hyp.stage_create(cfg, 0, 1, [w])
    del w
    x = torch.full((T, shape.hidden), 0.5, dtype=torch.bfloat16, device="cuda")
    y = torch.empty_like(x)
    for _ in range(2):
        stage.prefill(x, lens, y)
    stage.profile(["gemm_gateup"])
    for _ in range(3):
        stage.prefill(x, lens, y)
    torch.cuda.synchronize()
    ms, n = stage.profile_read("gemm_gateup")
    stage.profile([])
    stage.destroy()
    return 2.0 * T * 2 * shape.ffn_dim * shape.hidden / (ms / n * 1e-3) / 1e12


def library_gemm_tflops(wl):
    """A yardstick, not a path of the stage: the vendor BLAS (what torch.matmul dispatches to) on the four
    projection shapes of the timed prefill, same Gaussian bf16 operands, plain bf16 output and none of the
    fused epilogues - what a tuned hand-written assembly GEMM reaches on this device and this data."""
    import torch
    shape = wl.shape
    T = sum(wl.lengths())
    H, I, qd, kvd = shape.hidden, shape.ffn_dim, shape.q_dim, shape.kv_dim
    res = {}
    for name, (N, K) in {"gemm_qkv": (qd + 2 * kvd, H), "gemm_o": (H, qd), "gemm_gateup": (2 * I, H), "gemm_down": (H, I)}.items():
        a = device_normal((T, K), wl.seed + 7)
        b = (device_normal((N, K), wl.seed + 8).float() * 0.02).to(torch.bfloat16)
        for _ in range(2):
            c = a @ b.t()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        for _ in range(4):
            c = a @ b.t()
        ev[1].record()
        torch.cuda.synchronize()
        res[name] = 2.0 * T * N * K / (ev[0].elapsed_time(ev[1]) / 4 * 1e-3) / 1e12
        del a, b, c
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD,
                    choices=[k for k in synth.WORKLOADS if k not in ("c1_tiny_f32", "c2_layer_prefill")])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the measured ceilings and the other configurations (profiling runs: only the workload's kernels)")
    ap.add_argument("--layers", type=int, default=0, help="override the block count (counter runs on a shorter stage)")
    ap.add_argument("--decode-steps", type=int, default=-1, help="override the number of decode steps")
    ap.add_argument("--no-graph", action="store_true", help="launch decode kernels one by one (for counter runs)")
    ap.add_argument("--paged", action="store_true", help="keep the KV cache in 128-key pages behind a shuffled page table")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also run one 256 MiB device copy, the known-size reference for FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one stage on ONE GPU: a stage is the unit the pipeline places on a single "
              "device, and the library has no multi-GPU path. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2511_14450_amd as hyp

    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(1)
    wl = synth.WORKLOADS[args.workload]
    overridden = args.layers > 0 or args.decode_steps >= 0
    if overridden:
        wl = dataclasses.replace(wl, n_layers=args.layers if args.layers > 0 else wl.n_layers,
                                 decode_steps=args.decode_steps if args.decode_steps >= 0 else wl.decode_steps)
    r = run_workload(wl, args.steps, args.warmup, no_graph=args.no_graph, traffic_calibration=args.traffic_calibration,
                     paged=args.paged)
    if overridden:
        r["config"]["workload"] += " (overridden)"
    out = {
        "metric": "stage tokens/sec (prefill & decode) per MI355X",
        "value": r.pop("value"),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": r.pop("ms_per_step"),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
    }
    out.update(r)
    if not args.no_extras:
        # what this device delivers at best, measured in the same run: the MFMA pipes from
        # registers (Gaussian operands make the chip clock down; constants do not) and a
        # plain streaming read
        out["measured_ceilings"] = {
            "mfma_bf16_gaussian_operands_tflops": hyp.hyp_measure_mfma_ceiling(True),      # 16x16x32, the GEMM's instruction
            "mfma_bf16_constant_operands_tflops": hyp.hyp_measure_mfma_ceiling(False),
            "mfma_bf16_32x32x16_gaussian_operands_tflops": hyp.hyp_measure_mfma_ceiling(True, True),
            "hbm_stream_read_gbs": hyp.hyp_measure_hbm_read_ceiling(4),
            "gemm_gateup_kernel_constant_operands_tflops": gemm_constant_operands_tflops(wl),
            "library_gemm_same_shapes_gaussian_operands_tflops": library_gemm_tflops(wl),
        }
        # the same fractions against what the device was measured to deliver (the datasheet figures stay the headline)
        mc = out["measured_ceilings"]
        gemm = [k for k in out["kernels"] if k["kernel"].startswith("gemm_")]
        out["fractions_of_measured_ceilings"] = {
            "decode_step_of_hbm_stream_read": out["decode_frac_of_hbm_peak"] * PEAK_HBM_GBS / mc["hbm_stream_read_gbs"]
            if out.get("decode_frac_of_hbm_peak") else None,
            "prefill_gemm_kernels_of_mfma_gaussian": {k["kernel"]: k["achieved"] / mc["mfma_bf16_gaussian_operands_tflops"] for k in gemm},
        }
        progress("measured ceilings done")
        if not overridden:
            # the other configurations, each timed over 1 warm-up + 2 steps (figures, not the headline value)
            others = [k for k in ("c3_stage10", "c4_decode_heavy", "n4_llama3_stage8", "c5_long") if k != args.workload]
            if args.workload != DEFAULT_WORKLOAD:
                others.remove(DEFAULT_WORKLOAD)  # the 20-block stage only as the headline
            out["other_configs"] = [brief(run_workload(synth.WORKLOADS[k], 2, 1)) for k in others]
            out["other_configs"].append(brief(run_workload(synth.WORKLOADS["c4_decode_heavy"], 2, 1, paged=True)))
            out["other_configs"].append(prefill_only_line("c2_layer_prefill"))
    if not args.no_cpu_baseline:
        progress("timing the CPU oracle on its sample")
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
