"""Length sweeps in the shape of the paper's own tables (Sec. 4.1 decode table,
Sec. 4.2 causal prefill table): uniform lengths, Llama-3-8B attention shape
(32 query heads, 8 KV heads, head_dim 128 or, with --head-dim 256, the paper's
second head size), page size 256.

    python -m paper_2604_15464_amd.sweep [--decode] [--prefill] [--steps K] [--max-len L] [--head-dim D]

Decode: n = 128 sequences, q_len 1, identical context length 512 ... 32768;
reports the step latency and the algorithmic GB/s (the paper's byte formula
with decimal units).  Prefill: one sequence of 512 ... 32768 tokens, causal,
no cached context; reports latency and TFLOP/s with exact causal FLOPs,
then the same lengths without the causal mask (4*s*s*Hq*D FLOPs).
One JSON line per point on stdout, a table on stderr.  Synthetic N(0,1) data.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

from . import rpa
from . import workloads as W

LENGTHS = (512, 1024, 2048, 4096, 8192, 16384, 32768)


def time_workload(wl, steps, warmup, causal=True, kv_scales=None):
    import torch

    dev = torch.device("cuda:0")
    x = W.materialize(wl, dev, poison=False, kv_scales=kv_scales)
    table = torch.from_numpy(wl.page_table).to(dev)
    ctx = rpa.RaggedPagedAttention.for_workload(wl, causal=causal, kv_scales=kv_scales)
    out = torch.empty_like(x["q"])

    def call():
        ctx.update_and_attend(x["q"], x["k_new"], x["v_new"], x["k_pages"], x["v_pages"], table,
                              wl.cu_q_lens, wl.kv_lens, wl.sm_scale, out=out)

    # the requested warm-up, then more until the GPU has been busy for 50 ms: short
    # rows would otherwise be timed while the clocks of an idle GPU still settle
    t_w = time.perf_counter()
    done = 0
    while done < warmup or time.perf_counter() - t_w < 0.05:
        call()
        done += 1
        if done % 32 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        call()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    ctx.profile_enable(True)
    for _ in range(steps):
        call()
    torch.cuda.synchronize()
    prof = ctx.profile_read()
    info = ctx.plan_info()
    ctx.close()
    del x, table, out
    torch.cuda.empty_cache()
    n = max(1, prof["calls"])
    return dt, {k: prof[k] / n for k in ("narrow_ms", "wide_ms", "combine_ms")}, info


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--decode", action="store_true")
    ap.add_argument("--prefill", action="store_true")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--max-len", type=int, default=32768)
    ap.add_argument("--head-dim", type=int, default=128, choices=(64, 128, 256))
    ap.add_argument("--kv-fp8", action="store_true",
                    help="decode table with the 8-bit (E4M3) KV cache; bytes counted at one byte per cached element")
    args = ap.parse_args()
    d = args.head_dim
    if args.kv_fp8:
        args.decode, args.prefill = True, False      # the 8-bit cache is built for the decode case
    kv_scales = (1.0 / 64.0, 1.0 / 32.0) if args.kv_fp8 else None
    both = not (args.decode or args.prefill)
    rows = []
    if args.decode or both:
        for c in LENGTHS:
            if c > args.max_len:
                break
            wl = W.uniform(128, 1, c + 1, d=d)
            dt, k, info = time_workload(wl, args.steps, args.warmup, kv_scales=kv_scales)
            gbps = wl.algorithmic_bytes(kv_fp8=args.kv_fp8) / dt / 1e9
            rec = {"sweep": "decode_fp8_cache" if args.kv_fp8 else "decode", "head_dim": d, "n": 128, "context": c,
                   "page_size": 256,
                   "latency_us": round(dt * 1e6, 1),
                   "GBps": round(gbps, 1), "pct_of_8TBps": round(gbps / 80.0, 2),
                   "narrow_kernel_us": round(k["narrow_ms"] * 1e3, 1), "combine_kernel_us": round(k["combine_ms"] * 1e3, 1),
                   "units": info["num_narrow_units"], "bins": info["num_narrow_bins"]}
            rows.append(rec)
            print(json.dumps(rec), flush=True)
    if args.prefill or both:
        for s in LENGTHS:
            if s > args.max_len:
                break
            wl = W.uniform(1, s, s, d=d)
            dt, k, info = time_workload(wl, args.steps, args.warmup)
            tf = wl.algorithmic_flops() / dt / 1e12
            rec = {"sweep": "prefill_causal", "head_dim": d, "n": 1, "seq_len": s, "page_size": 256,
                   "latency_us": round(dt * 1e6, 1),
                   "TFLOPs": round(tf, 1), "pct_of_2500": round(tf / 25.0, 2),
                   "wide_kernel_us": round(k["wide_ms"] * 1e3, 1), "combine_kernel_us": round(k["combine_ms"] * 1e3, 1),
                   "units": info["num_wide_units"], "wide_rows": info["wide_rows"], "max_splits": info["max_splits"]}
            rows.append(rec)
            print(json.dumps(rec), flush=True)
    if args.prefill or both:
        for s in LENGTHS:
            if s > args.max_len:
                break
            wl = W.uniform(1, s, s, d=d)
            dt, k, info = time_workload(wl, args.steps, args.warmup, causal=False)
            tf = 4.0 * wl.num_q_heads * wl.head_dim * s * s / dt / 1e12  # every (query, key) pair is visible
            rec = {"sweep": "prefill_noncausal", "head_dim": d, "n": 1, "seq_len": s, "page_size": 256,
                   "latency_us": round(dt * 1e6, 1), "TFLOPs": round(tf, 1), "pct_of_2500": round(tf / 25.0, 2),
                   "wide_kernel_us": round(k["wide_ms"] * 1e3, 1), "combine_kernel_us": round(k["combine_ms"] * 1e3, 1),
                   "units": info["num_wide_units"], "wide_rows": info["wide_rows"], "max_splits": info["max_splits"]}
            rows.append(rec)
            print(json.dumps(rec), flush=True)
    for r in rows:
        print("  ".join(f"{k}={v}" for k, v in r.items()), file=sys.stderr)


if __name__ == "__main__":
    main()
