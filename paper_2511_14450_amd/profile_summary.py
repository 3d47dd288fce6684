#!/usr/bin/env python3
"""Turn rocprofv3 CSV output of `bench.py` into the short text summaries kept under profiles/.

  kernel stats :  python -m paper_2511_14450_amd.profile_summary stats  <dir>/<name>_kernel_stats.csv
  HBM traffic  :  python -m paper_2511_14450_amd.profile_summary traffic <fetch>_counter_collection.csv <write>_counter_collection.csv
                  [--json profiles/traffic_c5_long.json --workload c5_long]
  MFMA / waits :  python -m paper_2511_14450_amd.profile_summary counters <dir>/<name>_counter_collection.csv

FETCH_SIZE / WRITE_SIZE are reported by rocprofv3 in KiB per dispatch; both are scaled by
what the same counter reads for the 256 MiB device copy that `bench.py --traffic-calibration`
runs (the scale factors are printed).
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import pathlib
import re
import sys

# kernel class, as bench.py and hyp_stage.h name it, of every kernel of the MFMA path.  The GEMM
# kernels carry their class as their last template argument (a hyp_kernel_class_t), so the O and
# down projections, which share an epilogue, have different names in a trace.
CLASS_BY_ID = {1: "gemm_qkv", 3: "gemm_o", 4: "gemm_gateup", 5: "gemm_down",
               6: "gemv_qkv", 9: "gemv_o", 10: "gemv_gateup", 12: "gemv_down"}
CLASS_BY_NAME = [(r"k_attn_prefill", "attn_prefill"), (r"k_attn_decode_merge", "attn_decode_merge"),
                 (r"k_attn_decode", "attn_decode"), (r"k_rstd", "add_norm"), (r"k_add_norm", "add_norm"),
                 (r"k_dec_begin", "dec_begin")]


def short(name: str) -> str:
    m = re.search(r"(k_\w+)(<[^>]*>)?", name)
    return (m.group(1) + (m.group(2) or "")) if m else name.split("(")[0][-48:]


def classify(row) -> str:
    n = short(row["Kernel_Name"])
    m = re.match(r"k_(gemm|dec_gemv)<.*?(\d+)>$", n)
    if m:
        return CLASS_BY_ID.get(int(m.group(2)), n)
    for pat, cls in CLASS_BY_NAME:
        if re.search(pat, n):
            return cls
    return n


def stats(path):
    rows = list(csv.DictReader(open(path)))
    print(f"{'kernel':44s} {'calls':>7s} {'avg_us':>10s} {'total_ms':>10s} {'pct':>6s}")
    for r in rows:
        if float(r["Percentage"]) < 0.05:
            continue
        print(f"{short(r['Name']):44s} {r['Calls']:>7s} {float(r['AverageNs']) / 1e3:10.1f} "
              f"{float(r['TotalDurationNs']) / 1e6:10.1f} {float(r['Percentage']):6.2f}")


def per_class(path, counter):
    agg = collections.defaultdict(list)
    copy = []
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        v = float(r["Counter_Value"])
        name = r["Kernel_Name"]
        if "copyBuffer" in name:
            copy.append((v, name))
        agg[classify(r)].append(v)
    return agg, copy


def traffic(fetch_csv, write_csv, out_json, workload):
    f, fcopy = per_class(fetch_csv, "FETCH_SIZE")
    w, wcopy = per_class(write_csv, "WRITE_SIZE")
    ref_kib = 256 * 1024.0
    # the calibration copy is the largest copy-like dispatch
    fscale = ref_kib / max(v for v, _ in fcopy) if fcopy else 1.0
    wscale = ref_kib / max(v for v, _ in wcopy) if wcopy else 1.0
    print(f"calibration: 256 MiB copy read as FETCH_SIZE={max(v for v, _ in fcopy) if fcopy else float('nan'):.0f} KiB "
          f"(scale {fscale:.4f}), WRITE_SIZE={max(v for v, _ in wcopy) if wcopy else float('nan'):.0f} KiB (scale {wscale:.4f})")
    print(f"{'kernel class':36s} {'launches':>8s} {'fetch MiB':>10s} {'write MiB':>10s}")
    result = {}
    for cls in sorted(set(f) | set(w)):
        if not cls.startswith(("gemm", "gemv", "attn", "k_gemm", "k_dec", "add_norm", "dec_")):
            continue
        cls_out = cls
        fb = sum(f.get(cls, [0])) / max(len(f.get(cls, [1])), 1) * fscale * 1024
        wb = sum(w.get(cls, [0])) / max(len(w.get(cls, [1])), 1) * wscale * 1024
        print(f"{cls_out:36s} {len(f.get(cls, [])):8d} {fb / 2**20:10.1f} {wb / 2**20:10.1f}")
        result[cls_out] = fb + wb
    if out_json:
        sys.path.insert(0, str(pathlib.Path(__file__).resolve().parents[1]))
        import bench
        json.dump({"workload": workload, "sources_sha256": bench.kernel_sources_digest(),
                   "unit": "bytes (FETCH_SIZE + WRITE_SIZE, scaled by the copy calibration)",
                   "hbm_bytes_per_launch": result}, open(out_json, "w"), indent=1)


def counters(path):
    """MFMA busy / wait / LDS conflict ratios per kernel from one --pmc run with
    SQ_VALU_MFMA_BUSY_CYCLES SQ_WAVE_CYCLES SQ_WAIT_ANY SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE GRBM_GUI_ACTIVE."""
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        agg[short(r["Kernel_Name"]) + " grid " + r["Grid_Size"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    print(f"{'kernel':34s} {'cycles/XCD':>11s} {'MFMA busy':>10s} {'wave wait':>10s} {'LDS conflict':>12s}")
    for k, v in agg.items():
        if not re.match(r"k_(gemm|attn|dec_gemv|mfma_only|add_norm|rstd)", k):
            continue
        a = {c: sum(x) / len(x) for c, x in v.items()}
        cyc = a["GRBM_GUI_ACTIVE"] / 8
        busy = a["SQ_VALU_MFMA_BUSY_CYCLES"] / 1024 / cyc
        wait = a["SQ_WAIT_ANY"] / a["SQ_WAVE_CYCLES"]
        conf = a["SQ_LDS_BANK_CONFLICT"] / a["SQ_LDS_IDX_ACTIVE"] if a["SQ_LDS_IDX_ACTIVE"] else 0.0
        print(f"{k:34s} {cyc:11.0f} {busy:10.3f} {wait:10.3f} {conf:12.3f}")


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("mode", choices=["stats", "traffic", "counters"])
    ap.add_argument("files", nargs="+")
    ap.add_argument("--json")
    ap.add_argument("--workload", default="c5_long")
    a = ap.parse_args()
    if a.mode == "stats":
        stats(a.files[0])
    elif a.mode == "counters":
        counters(a.files[0])
    else:
        traffic(a.files[0], a.files[1], a.json, a.workload)
