"""Sweep of the Llama-shaped SR decode step over context length, batch, rank and selection budget.

Runs `bench.py` once per point (a fresh process each, so that every point starts from an empty device) and
collects the JSON lines.  Usage, from the repository root on a machine with the GPU:

    python -m paper_2503_18893_amd.sweep --L 65536 --out sweep_L64k.jsonl
    python -m paper_2503_18893_amd.sweep --table sweep_L16k.jsonl sweep_L32k.jsonl ...   # markdown table only

Every point: 32 layers (8 groups of G = 4), H_kv = 8, H_q = 32, d_h = 128, bf16; SR tokens/s, dense tokens/s
(on as many resident layer caches as fit), speedup, and the HBM rates of the score, gather-attend and dense
kernels from algorithmic bytes.
"""
from __future__ import annotations

import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_point(L, batch, r, kfrac, steps, timeout_s):
    k = max(1, int(round(L * kfrac)))
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "llama_full", "--L", str(L), "--batch",
           str(batch), "--r", str(r), "--k", str(k), "--no-cpu", "--no-factorize", "--no-landmark", "--no-graph",
           "--steps", str(steps), "--warmup", "1"]
    t0 = time.perf_counter()
    try:
        res = subprocess.run(cmd, capture_output=True, text=True, timeout=timeout_s)
    except subprocess.TimeoutExpired:
        return {"L": L, "batch": batch, "r": r, "k": k, "kfrac": kfrac, "error": "timeout"}
    rec = {"L": L, "batch": batch, "r": r, "k": k, "kfrac": kfrac, "wall_s": round(time.perf_counter() - t0, 1)}
    lines = [ln for ln in res.stdout.strip().splitlines() if ln.startswith("{")]
    if res.returncode != 0 or not lines:
        rec["error"] = (res.stderr.strip().splitlines() or ["no output"])[-1][:200]
        return rec
    d = json.loads(lines[-1])
    dense = d.get("dense_baseline") or {}
    rec.update(sr_tokens_per_s=d["value"], sr_ms=d["ms_per_step"], dense_tokens_per_s=dense.get("tokens_per_s"),
               dense_ms=dense.get("ms_per_step"), dense_GBps=dense.get("GBps"), dense_note=dense.get("note"),
               speedup=d.get("speedup_vs_dense"), score_GBps=d["stages"]["score"].get("kernel_GBps"),
               gather_GBps=d["stages"]["gather_attend"].get("kernel_GBps"),
               topk_ms=d["stages"]["topk"]["ms_per_layer"],
               absorbed_tokens_per_s=(d.get("absorbed") or {}).get("tokens_per_s"),
               q4_tokens_per_s=(d.get("quantized") or {}).get("tokens_per_s"))
    return rec


def table(records):
    out = ["| L | batch | r | k | SR tok/s | dense tok/s | SR/dense | score TB/s | gather TB/s | dense TB/s | "
           "absorbed tok/s | 4-bit absorbed tok/s |",
           "|---:|---:|---:|---:|---:|---:|---:|---:|---:|---:|---:|---:|"]

    def tb(x):
        return "-" if x is None else f"{x / 1000:.2f}"

    def tk(x):   # the two absorbed forms are extras of bench.py; records made before they existed have none
        return "-" if x is None else f"{x:.0f}"

    for r in records:
        if "error" in r:
            out.append(f"| {r['L']} | {r['batch']} | {r['r']} | {r['k']} | {r['error']} | | | | | | | |")
            continue
        dn = "" if not r.get("dense_note") or r["dense_note"].startswith("all") else "*"
        dense_tok = "-" if r["dense_tokens_per_s"] is None else f"{r['dense_tokens_per_s']:.0f}{dn}"
        out.append(f"| {r['L']} | {r['batch']} | {r['r']} | {r['k']} | {r['sr_tokens_per_s']:.0f} | "
                   f"{dense_tok} | {r['speedup'] if r['speedup'] is not None else '-'} | "
                   f"{tb(r['score_GBps'])} | {tb(r['gather_GBps'])} | {tb(r['dense_GBps'])} | "
                   f"{tk(r.get('absorbed_tokens_per_s'))} | {tk(r.get('q4_tokens_per_s'))} |")
    return "\n".join(out)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--L", type=int, nargs="+", default=[16384, 32768, 65536, 131072])
    ap.add_argument("--batch", type=int, nargs="+", default=[1, 4, 16, 32])
    ap.add_argument("--r", type=int, nargs="+", default=[256, 512, 768])
    ap.add_argument("--kfrac", type=float, nargs="+", default=[0.015, 0.03, 0.06, 0.125])
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--timeout", type=int, default=240, help="seconds per point")
    ap.add_argument("--out", default=None, help="append one JSON record per point to this file")
    ap.add_argument("--table", nargs="+", default=None, help="only print the table of these record files")
    args = ap.parse_args()
    if args.table:
        recs = [json.loads(ln) for f in args.table for ln in open(f) if ln.strip()]
        print(table(recs))
        return
    recs = []
    for L in args.L:
        for batch in args.batch:
            for r in args.r:
                for kf in args.kfrac:
                    rec = run_point(L, batch, r, kf, args.steps, args.timeout)
                    recs.append(rec)
                    print(json.dumps(rec), flush=True)
                    if args.out:
                        with open(args.out, "a") as f:
                            f.write(json.dumps(rec) + "\n")
    print(table(recs))


if __name__ == "__main__":
    main()
