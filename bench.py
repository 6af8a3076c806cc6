#!/usr/bin/env python3
"""Benchmark of the ragged paged attention hot path on one MI355X.

One "step" is one call of rpa_update_and_attend (host partition + work-list
upload + fused cache write + attention + split merge) on a batch that is
already resident in HBM.  The headline line is the decode workload
(256 sequences, q_len 1, kv_len ~ U[512, 4096], Llama-3-8B attention shape)
reported as achieved HBM GB/s; the prefill workload (8 x 2048 causal) is
reported in the same JSON line under "prefill" as attention TFLOP/s, the
mixed batch (128 decode + 4 chunked prefills) under "mixed" as time per call.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Prints exactly one JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix, vendor figure


def log(*a):
    print(*a, file=sys.stderr, flush=True)


MIN_WARMUP_CALLS = 100
MIN_WARMUP_S = 0.05
IDLE_BEFORE_BLOCK_S = 1.0
FLOOR = {"calls": MIN_WARMUP_CALLS, "idle_s": IDLE_BEFORE_BLOCK_S, "blocks_run": 0}
KV_SCALES = (1.0 / 64.0, 1.0 / 32.0)   # 8-bit cache block: N(0,1) / scale stays inside +-448


def time_steps(ctx, x, table, wl, steps, warmup):
    """Returns (seconds for `steps` whole steps, per-kernel milliseconds of a
    second pass of `steps` steps).  The first pass is the throughput figure and
    carries no instrumentation; the second attaches a start and a stop HIP event
    to every kernel dispatch (on the stream the kernels run on), which costs a
    few microseconds per step and therefore stays out of the first."""
    import torch
    # Every block starts from the state the first one finds: an idle GPU.  Right after
    # another block's load the chip runs the next one 1-3 % slower for hundreds of
    # calls (mixed batch: 409-415 us behind the decode or prefill block, 398-404 us
    # alone or after a second of idle), which would be the neighbour's footprint.
    if FLOOR["idle_s"] > 0 and FLOOR["blocks_run"] > 0:
        torch.cuda.synchronize()
        time.sleep(FLOOR["idle_s"])
    FLOOR["blocks_run"] += 1

    def call():
        ctx.update_and_attend(x["q"], x["k_new"], x["v_new"], x["k_pages"], x["v_pages"], table,
                              cu, kv, wl.sm_scale, out=out)

    cu, kv = wl.cu_q_lens, wl.kv_lens
    out = torch.empty_like(x["q"])
    # The requested warm-up, then more until the GPU has been busy for at least
    # MIN_WARMUP_CALLS calls and MIN_WARMUP_S seconds: the clocks of an idle GPU take
    # some tens of milliseconds of load to settle, and the first calls of a short
    # warm-up run up to 10 % slower than the steady state that is being measured.
    t_w = time.perf_counter()
    done = 0
    while done < warmup or (FLOOR["calls"] > 0 and (done < FLOOR["calls"] or time.perf_counter() - t_w < MIN_WARMUP_S)):
        call()
        done += 1
        if done % 32 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        call()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ctx.profile_enable(True)
    for _ in range(steps):
        call()
    torch.cuda.synchronize()
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    return dt, prof, out


def stream_copy(ctx, nbytes, reps):
    """The library's plain copy kernel on `nbytes` bytes: the known-size
    workload the HBM counters are calibrated against, and the streaming rate
    this box reaches without any attention work."""
    import torch

    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    ms = [ctx.copy_probe(dst, src) for _ in range(reps)]
    ok = bool(torch.equal(dst, src))
    best = min(ms[1:] or ms)
    return {"bytes": nbytes, "reps": reps, "ms": round(best, 5), "read_plus_write_GBps": round(2 * nbytes / best / 1e6, 1),
            "verified": ok}


def load_traffic(workload, kernel):
    """HBM bytes per launch from the tracked counter summary (two rocprofv3 --pmc
    runs, FETCH_SIZE and WRITE_SIZE): a figure of those runs, not of this one."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f)[workload][kernel]["hbm_bytes_per_launch"]
    except Exception:
        return None


TRAFFIC_SOURCE = ("profiles/hbm_traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of the same workloads, "
                  "scaled by the plain copy kernel; replayed from that file, not measured by this run")


def narrow_part(wl):
    """The sequences of a batch that the narrow kernel serves by default (at most
    one narrow tile of query tokens), as a workload of their own: only its
    lengths are used, for byte counts."""
    from paper_2604_15464_amd import workloads as W
    hg = wl.num_q_heads // wl.num_kv_heads
    keep = wl.q_lens <= 16 // hg
    return W.Workload(wl.name + "[narrow]", wl.seed, wl.num_q_heads, wl.num_kv_heads, wl.head_dim, wl.page_size,
                      wl.num_pages, wl.q_lens[keep], wl.kv_lens[keep], wl.page_table[keep])


def cpu_baseline(wl, budget_s=15.0):
    """Time the CPU oracle, as it stands, on a bounded sample of the workload:
    the first sequences of the batch with their own page pool."""
    import numpy as np
    import torch
    from oracle import rpa_oracle as O
    from paper_2604_15464_amd import workloads as W

    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1

    def sample(n):
        rng = np.random.default_rng(wl.seed + 7)
        q, kv = wl.q_lens[:n], wl.kv_lens[:n]
        pages = int(W.pages_needed(kv, wl.page_size).sum())
        return W.Workload(f"{wl.name}[:{n}]", wl.seed, wl.num_q_heads, wl.num_kv_heads, wl.head_dim,
                          wl.page_size, pages, q, kv, W.make_page_table(kv, wl.page_size, pages, rng))

    def run(sub):
        x = {k: W.bits(v) for k, v in W.materialize(sub, "cpu", poison=False).items()}
        t0 = time.perf_counter()
        O.update_and_attend(x["q"], x["k_new"], x["v_new"], x["k_pages"], x["v_pages"], sub.page_table,
                            sub.cu_q_lens, sub.kv_lens, sub.num_seqs, sub.sm_scale)
        return time.perf_counter() - t0

    probe = sample(min(4, wl.num_seqs))
    t_probe = run(probe)
    per_byte = t_probe / probe.algorithmic_bytes()
    n = wl.num_seqs
    while n > 4 and sample(n).algorithmic_bytes() * per_byte > budget_s:
        n //= 2
    sub = sample(n)
    times = [run(sub)]
    while sum(times) < 0.7 * budget_s and len(times) < 32:  # a cheap sample is repeated, not enlarged
        times.append(run(sub))
    return sub, sum(times) / len(times), len(times), cores


def decode_block(args, rpa, W, torch, dev, wl):
    """The headline block: config 2, decode-only."""
    x = W.materialize(wl, dev, poison=False)
    table = torch.from_numpy(wl.page_table).to(dev)
    ctx = rpa.RaggedPagedAttention.for_workload(wl)
    copy = stream_copy(ctx, args.copy_bytes - args.copy_bytes % 16, 4) if args.copy_bytes >= 16 else None
    dt, prof, _ = time_steps(ctx, x, table, wl, args.steps, args.warmup)
    info = ctx.plan_info()
    ctx.close()
    ms_per_step = dt / args.steps * 1e3
    nbytes = wl.algorithmic_bytes()
    value = nbytes / (dt / args.steps) / 1e9
    narrow_ms = prof["narrow_ms"] / max(1, prof["calls"])
    achieved = nbytes / (narrow_ms * 1e-3) / 1e9
    log(f"decode: {ms_per_step * 1e3:.1f} us/step, kernel {narrow_ms * 1e3:.1f} us, combine "
        f"{prof['combine_ms'] / max(1, prof['calls']) * 1e3:.1f} us, plan {info}")
    result = {
        "metric": "decode HBM GB/s",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "decode-only: 256 seqs, q_len 1, kv_len~U[512,4096], Hq32 Hkv8 D128 page16 "
                               "(Llama-3-8B attention shape), fused KV write + attention",
                   "name": wl.name, "algorithmic_bytes_per_step": nbytes,
                   "variant": rpa.VARIANT_NAMES[info["variant"]], "units": info["num_narrow_units"],
                   "bins": info["num_narrow_bins"], "max_splits": info["max_splits"]},
        "pct_of_peak_hbm": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "roofline": {"kernel": "rpa_narrow_kernel<128>", "bound": "hbm", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": load_traffic(wl.name, "rpa_narrow_kernel"), "traffic_source": TRAFFIC_SOURCE,
                     "avg_kernel_ms": round(narrow_ms, 5)},
        "warmup_effective": f"max(--warmup, {FLOOR['calls']} calls, {MIN_WARMUP_S} s) before every timed block; "
                            f"{FLOOR['idle_s']} s of idle GPU before every block but the first",
    }
    return result, dt, copy


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true",
                    help="profiling runs only: skip the headline decode block (value is then null), so that every "
                         "dispatch of a kernel in the run belongs to one block")
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--no-mixed", action="store_true")
    ap.add_argument("--no-fp8", action="store_true")
    ap.add_argument("--min-warmup-calls", type=int, default=MIN_WARMUP_CALLS,
                    help="floor on the warm-up calls of every timed block (counter-collection runs lower it)")
    ap.add_argument("--idle-before-block", type=float, default=IDLE_BEFORE_BLOCK_S,
                    help="seconds of idle GPU before every timed block but the first, so that each starts "
                         "from the state the first finds (0 = none)")
    ap.add_argument("--only", default="", help="comma list of blocks to run besides the headline decode block: "
                    "prefill,mixed,fp8,long_decode (default: all)")
    ap.add_argument("--copy-bytes", type=int, default=1 << 30,
                    help="size of the plain copy that calibrates HBM counters (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU; --gpus must be 1 (no collectives, no sharding in this path).")
        sys.exit(2)
    if args.steps < 1 or args.steps > 1024:
        log("bench.py: --steps must be in 1..1024")
        sys.exit(2)

    import torch
    from paper_2604_15464_amd import rpa
    from paper_2604_15464_amd import workloads as W

    FLOOR["calls"] = max(0, args.min_warmup_calls)
    FLOOR["idle_s"] = max(0.0, args.idle_before_block)
    only = set(filter(None, args.only.split(",")))
    if only - {"prefill", "mixed", "fp8", "long_decode", "none"}:
        log("bench.py: --only takes prefill, mixed, fp8, long_decode, none")
        sys.exit(2)

    def wanted(block, off):
        return not off and (not only or block in only)

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    # ---- decode (headline) ----------------------------------------------------
    wl = W.config(2)
    copy = None
    if args.no_decode:
        ctx0 = rpa.RaggedPagedAttention.for_workload(W.config(1))
        copy = stream_copy(ctx0, args.copy_bytes - args.copy_bytes % 16, 4) if args.copy_bytes >= 16 else None
        ctx0.close()
        dt = float("nan")
        result = {"metric": "decode HBM GB/s", "value": None, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
                  "warmup": args.warmup, "higher_is_better": True, "data": "synthetic", "dtype": "bf16",
                  "config": {"workload": "headline decode block skipped (--no-decode)", "name": None}}
    else:
        result, dt, copy = decode_block(args, rpa, W, torch, dev, wl)
    if copy is not None:
        result["stream_copy"] = copy
    torch.cuda.empty_cache()

    # ---- mixed batch (decode + chunked prefill in one call) ---------------------------
    if wanted("mixed", args.no_mixed):
        wl4 = W.config(4)
        x4 = W.materialize(wl4, dev, poison=False)
        table4 = torch.from_numpy(wl4.page_table).to(dev)
        ctx4 = rpa.RaggedPagedAttention.for_workload(wl4)
        dt4, prof4, _ = time_steps(ctx4, x4, table4, wl4, args.steps, args.warmup)
        info4 = ctx4.plan_info()
        ctx4.close()
        n4 = max(1, prof4["calls"])
        us4 = dt4 / args.steps * 1e6
        log(f"mixed: {us4:.1f} us/step, narrow {prof4['narrow_ms'] / n4 * 1e3:.1f} us, wide "
            f"{prof4['wide_ms'] / n4 * 1e3:.1f} us, combine {prof4['combine_ms'] / n4 * 1e3:.1f} us, plan {info4}")
        result["mixed"] = {
            "metric": "mixed-batch step time", "value": round(us4, 1), "unit": "us", "higher_is_better": False,
            "steps": args.steps,
            "config": {"workload": "mixed: 128 decode seqs kv_len~U[256,8192] + 4 chunked prefills of 512 tokens on "
                                   "contexts 1K/2K/4K/8K, shuffled, Hq32 Hkv8 D128 page16",
                       "name": wl4.name, "algorithmic_bytes_per_step": wl4.algorithmic_bytes(),
                       "exact_causal_flops_per_step": wl4.algorithmic_flops(),
                       "kernels_side_by_side": bool(info4["concurrent"]),
                       "one_launch": info4["concurrent"] == 2},
            "GBps": round(wl4.algorithmic_bytes() / (dt4 / args.steps) / 1e9, 1),
            "TFLOPs": round(wl4.algorithmic_flops() / (dt4 / args.steps) / 1e12, 1),
            "kernel_ms": {"narrow": round(prof4["narrow_ms"] / n4, 5), "wide": round(prof4["wide_ms"] / n4, 5),
                          "combine": round(prof4["combine_ms"] / n4, 5)},
        }
        # The call's roof: its bytes at the HBM peak or its FLOPs at the MFMA peak,
        # whichever takes longer (narrow and wide workgroups run side by side).  When
        # one launch holds both kinds of workgroup (reported as the narrow time, the
        # wide time is then 0) the dominant kernel is that launch and its bytes are
        # the call's; as two kernels it is the narrow one: its own bytes (the
        # short-query sequences) over its own duration.
        b4, f4 = wl4.algorithmic_bytes(), wl4.algorithmic_flops()
        t_roof = max(b4 / (HBM_PEAK_GBPS * 1e9), f4 / (MFMA_BF16_PEAK_TFLOPS * 1e12))
        one4 = info4["concurrent"] == 2
        nb4 = b4 if one4 else narrow_part(wl4).algorithmic_bytes()
        ach4 = nb4 / (prof4["narrow_ms"] / n4 * 1e-3) / 1e9
        result["mixed"]["roofline"] = {
            "kernel": "rpa_mixed_kernel<128>" if one4 else "rpa_narrow_kernel<128>", "bound": "hbm",
            "achieved": round(ach4, 1), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(ach4 / HBM_PEAK_GBPS, 4), "algorithmic_bytes_of_kernel": nb4,
            "traffic": load_traffic(wl4.name, "call"), "traffic_source": TRAFFIC_SOURCE,
            "avg_kernel_ms": round(prof4["narrow_ms"] / n4, 5),
            "call_roof_us": round(t_roof * 1e6, 1), "call_frac_of_roof": round(t_roof / (dt4 / args.steps), 4)}
        del x4, table4
        torch.cuda.empty_cache()

    # ---- decode over the 8-bit (E4M3, per-tensor scale) cache ---------------------------
    if wanted("fp8", args.no_fp8):
        x8 = W.materialize(wl, dev, poison=False, kv_scales=KV_SCALES)
        table8 = torch.from_numpy(wl.page_table).to(dev)
        ctx8 = rpa.RaggedPagedAttention.for_workload(wl, kv_scales=KV_SCALES)
        dt8, prof8, _ = time_steps(ctx8, x8, table8, wl, args.steps, args.warmup)
        ctx8.close()
        n8 = max(1, prof8["calls"])
        b8 = wl.algorithmic_bytes(kv_fp8=True)
        log(f"decode, 8-bit cache: {dt8 / args.steps * 1e6:.1f} us/step, kernel {prof8['narrow_ms'] / n8 * 1e3:.1f} us")
        result["decode_fp8_cache"] = {
            "metric": "decode HBM GB/s, KV cache of E4M3 bytes", "value": round(b8 / (dt8 / args.steps) / 1e9, 1),
            "unit": "GB/s", "steps": args.steps, "ms_per_step": round(dt8 / args.steps * 1e3, 5),
            "config": {"workload": "the headline decode workload with rpa_shape.kv_fp8 = 1 (k_new / v_new bf16, "
                                   "quantised on the way in)", "algorithmic_bytes_per_step": b8,
                       "k_scale": KV_SCALES[0], "v_scale": KV_SCALES[1]},
            "speedup_over_bf16_cache": None if args.no_decode else round(dt / dt8, 3),
            "kernel_ms": {"narrow": round(prof8["narrow_ms"] / n8, 5), "combine": round(prof8["combine_ms"] / n8, 5)},
        }
        del x8, table8
        torch.cuda.empty_cache()

    # ---- long-context skewed decode (32 sequences of 32 K - 128 K positions, page 64) ------
    if wanted("long_decode", False):
        wl5 = W.config(5)
        x5 = W.materialize(wl5, dev, poison=False)
        table5 = torch.from_numpy(wl5.page_table).to(dev)
        ctx5 = rpa.RaggedPagedAttention.for_workload(wl5)
        dt5, prof5, _ = time_steps(ctx5, x5, table5, wl5, args.steps, args.warmup)
        info5 = ctx5.plan_info()
        ctx5.close()
        n5 = max(1, prof5["calls"])
        b5 = wl5.algorithmic_bytes()
        k5 = prof5["narrow_ms"] / n5
        log(f"long decode: {dt5 / args.steps * 1e6:.1f} us/step, kernel {k5 * 1e3:.1f} us, combine "
            f"{prof5['combine_ms'] / n5 * 1e3:.1f} us, plan {info5}")
        result["long_decode"] = {
            "metric": "decode HBM GB/s", "value": round(b5 / (dt5 / args.steps) / 1e9, 1), "unit": "GB/s",
            "steps": args.steps, "ms_per_step": round(dt5 / args.steps * 1e3, 5),
            "pct_of_peak_hbm": round(100.0 * b5 / (dt5 / args.steps) / 1e9 / HBM_PEAK_GBPS, 2),
            "config": {"workload": "long-context skewed decode: 32 seqs, q_len 1, kv_len log-uniform in [32768, 131072], "
                                   "Hq32 Hkv8 D128 page64", "name": wl5.name, "algorithmic_bytes_per_step": b5,
                       "units": info5["num_narrow_units"], "bins": info5["num_narrow_bins"],
                       "max_splits": info5["max_splits"]},
            "roofline": {"kernel": "rpa_narrow_kernel<128>", "bound": "hbm", "achieved": round(b5 / (k5 * 1e-3) / 1e9, 1),
                         "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(b5 / (k5 * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                         "traffic": load_traffic(wl5.name, "rpa_narrow_kernel"), "traffic_source": TRAFFIC_SOURCE,
                         "avg_kernel_ms": round(k5, 5)},
            "kernel_ms": {"narrow": round(k5, 5), "combine": round(prof5["combine_ms"] / n5, 5)},
        }
        del x5, table5
        torch.cuda.empty_cache()

    # ---- prefill (second half of the metric) -------------------------------------
    # Last of the GPU blocks: the one matrix-bound load of the run, kept from
    # running ahead of the memory-bound blocks (see the idle gap in time_steps).
    if wanted("prefill", args.no_prefill):
        wl3 = W.config(3)
        x3 = W.materialize(wl3, dev, poison=False)
        table3 = torch.from_numpy(wl3.page_table).to(dev)
        ctx3 = rpa.RaggedPagedAttention.for_workload(wl3)
        steps3 = args.steps
        dt3, prof3, _ = time_steps(ctx3, x3, table3, wl3, steps3, args.warmup)
        info3 = ctx3.plan_info()
        # what this box's matrix pipe sustains, measured right behind the timed steps
        # (launches of MFMAs alone on every CU, 5-8 ms each; the rate falls within
        # milliseconds of matrix load, so the last of four is the one reported)
        probe = [ctx3.mfma_probe(6000) for _ in range(4)]
        mfma_only_tf = probe[-1][1] / (probe[-1][0] * 1e-3) / 1e12
        ctx3.close()
        flops = wl3.algorithmic_flops()
        wide_ms = prof3["wide_ms"] / max(1, prof3["calls"])
        tf = flops / (dt3 / steps3) / 1e12
        tf_k = flops / (wide_ms * 1e-3) / 1e12
        log(f"prefill: {dt3 / steps3 * 1e6:.1f} us/step, kernel {wide_ms * 1e3:.1f} us, plan {info3}")
        result["prefill"] = {
            "metric": "prefill attention TFLOP/s", "value": round(tf, 1), "unit": "TFLOP/s",
            "steps": steps3, "ms_per_step": round(dt3 / steps3 * 1e3, 5),
            "config": {"workload": "prefill-only: 8 seqs x 2048 causal, Hq32 Hkv8 D128 page16, all K/V new",
                       "name": wl3.name, "exact_causal_flops_per_step": flops,
                       "algorithmic_bytes_per_step": wl3.algorithmic_bytes(), "units": info3["num_wide_units"]},
            "pct_of_peak_bf16_mfma": round(100.0 * tf / MFMA_BF16_PEAK_TFLOPS, 2),
            "roofline": {"kernel": "rpa_wide_kernel<128>", "bound": "mfma", "achieved": round(tf_k, 1),
                         "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(tf_k / MFMA_BF16_PEAK_TFLOPS, 4),
                         "traffic": load_traffic(wl3.name, "rpa_wide_kernel"), "traffic_source": TRAFFIC_SOURCE,
                         "avg_kernel_ms": round(wide_ms, 5)},
            "mfma_only": {"value": round(mfma_only_tf, 1), "unit": "TFLOP/s",
                          "frac_of_peak": round(mfma_only_tf / MFMA_BF16_PEAK_TFLOPS, 4),
                          "kernel_frac_of_it": round(tf_k / mfma_only_tf, 4),
                          "launches_TFLOPs": [round(fl / (ms * 1e-3) / 1e12, 1) for ms, fl in probe],
                          "what": "rpa_mfma_probe: bf16 32x32x16 MFMAs alone on pseudo-random operands, 8 waves on "
                                  "each CU, no memory traffic; four launches of 6000 steps, the last one reported"},
        }
        del x3, table3
        torch.cuda.empty_cache()

    # ---- CPU oracle baseline ---------------------------------------------------------
    if not args.no_cpu_baseline:
        sub, t_cpu, reps, cores = cpu_baseline(wl)   # on the headline workload, whether or not its GPU block ran
        result["cpu_baseline"] = {
            "value": round(sub.algorithmic_bytes() / t_cpu / 1e9, 4), "unit": "GB/s", "cores": cores,
            "kind": "oracle",
            "sample": f"fp64 numpy oracle on the first {sub.num_seqs} of the workload's {wl.num_seqs} sequences "
                      f"(own page pool, {sub.algorithmic_bytes() / 1e6:.0f} MB algorithmic), mean of {reps} runs of "
                      f"{t_cpu:.2f} s",
        }
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
