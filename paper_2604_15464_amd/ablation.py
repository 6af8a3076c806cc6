"""Bottleneck attribution by leaving a stage out (the method of the paper's
ablation tables, Sec. 4.3), on the two benchmark workloads.

    python -m paper_2604_15464_amd.ablation [--steps K]

Decode (256 seqs, kv_len ~ U[512, 4096]): the narrow kernel as is, without the
cache write, without the attention math (loads and stores stay) and without the
K/V loads: the three columns of the paper's decode ablation table.  Prefill
(8 x 2048): the wide kernel as is, without K/V loads, with loads only, without
the output store, without the cache write.  The switches exist only in the
measurement build of the library (librpa_ablate.so, the same sources compiled
with -DRPA_ABLATE), which this script loads; the product library has none.
Outputs of ablated runs are meaningless; every access stays in bounds.  Prints
one JSON line per variant and a table on stderr.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

from . import rpa
from . import workloads as W

DECODE = (("full", 0), ("without cache write (w/o KV update)", 2), ("without attention math (w/o FA)", 1),
          ("without K/V loads (w/o DMA)", 4))
PREFILL = (("full", 0), ("without K/V loads", 64), ("K/V loads only (no compute)", 128),
           ("without output store", 256), ("without cache write", 512),
           ("launch, Q fetch and barriers only", 64 + 128 + 256 + 512))


def run(wl, variants, kernel_key, steps, warmup):
    import torch

    dev = torch.device("cuda:0")
    x = W.materialize(wl, dev, poison=False)
    table = torch.from_numpy(wl.page_table).to(dev)
    ctx = rpa.RaggedPagedAttention.for_workload(wl, library=rpa.load_library(rpa.ABLATE_LIB_PATH))
    out = torch.empty_like(x["q"])

    def call():
        ctx.update_and_attend(x["q"], x["k_new"], x["v_new"], x["k_pages"], x["v_pages"], table,
                              wl.cu_q_lens, wl.kv_lens, wl.sm_scale, out=out)

    rows = []
    for name, bits in variants:
        ctx.set_options(ablate=bits)
        for _ in range(warmup):
            call()
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
        ctx.profile_enable(False)
        rec = {"workload": wl.name, "variant": name, "ablate": bits, "step_us": round(dt * 1e6, 1),
               "kernel_us": round(prof[kernel_key] / max(1, prof["calls"]) * 1e3, 1)}
        rows.append(rec)
        print(json.dumps(rec), flush=True)
    ctx.close()
    del x, table, out
    torch.cuda.empty_cache()
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=10)
    args = ap.parse_args()
    rows = run(W.config(2), DECODE, "narrow_ms", args.steps, args.warmup)
    rows += run(W.config(3), PREFILL, "wide_ms", args.steps, args.warmup)
    for r in rows:
        print(f"{r['workload']:24s} {r['variant']:36s} step {r['step_us']:8.1f} us   kernel {r['kernel_us']:8.1f} us",
              file=sys.stderr)


if __name__ == "__main__":
    main()
