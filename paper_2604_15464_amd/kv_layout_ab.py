"""A/B of the two cache layouts on the decode path: separate K and V pools
([P, ps, Hkv, D] each) against the merged pool ([P, ps, Hkv, 2, D], the paper's
"KV merge", Sec. 3.1.3), same data, same page table, runs interleaved.

    python -m paper_2604_15464_amd.kv_layout_ab [2,5,d256:4096,...] [--page-size 16]

A token "dN:C" is a uniform decode batch of N sequences of context C.
"""
import argparse
import time

import numpy as np
import torch

from . import rpa
from . import workloads as W


def _time(ctx, call, steps, warm):
    for _ in range(warm):
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
    p = ctx.profile_read()
    ctx.profile_enable(False)
    return dt * 1e6, p["narrow_ms"] / max(1, p["calls"]) * 1e3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("workloads", nargs="?", default="2,5")
    ap.add_argument("--page-size", type=int, default=16)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--rounds", type=int, default=4)
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    for tok in args.workloads.split(","):
        if tok[0] == "d":
            n, c = (int(v) for v in tok[1:].split(":"))
            wl = W.uniform(n, 1, c + 1, d=128, ps=args.page_size)
        else:
            wl = W.config(int(tok))
        x = W.materialize(wl, dev, poison=False)
        m = W.merge_pools(x)
        table = torch.from_numpy(np.ascontiguousarray(wl.page_table)).to(dev)
        out_a, out_b = torch.empty_like(x["q"]), torch.empty_like(x["q"])
        a = rpa.RaggedPagedAttention.for_workload(wl)
        b = rpa.RaggedPagedAttention.for_workload(wl, kv_merged=True)

        def call_a():
            a.update_and_attend(x["q"], x["k_new"], x["v_new"], x["k_pages"], x["v_pages"], table, wl.cu_q_lens,
                                wl.kv_lens, wl.sm_scale, out=out_a)

        def call_b():
            b.update_and_attend(m["q"], m["k_new"], m["v_new"], m["kv_pages"], None, table, wl.cu_q_lens, wl.kv_lens,
                                wl.sm_scale, out=out_b)

        ra, rb = [], []
        for _ in range(args.rounds):
            ra.append(_time(a, call_a, args.steps, args.steps))
            rb.append(_time(b, call_b, args.steps, args.steps))
        diff = (out_a.float() - out_b.float()).abs().max().item()
        print(f"{wl.name} page_size {wl.page_size}: max |merged - separate| = {diff:.3g}")
        gb = wl.algorithmic_bytes() / 1e9
        for name, rr in (("separate", ra), ("merged", rb)):
            rr = np.array(rr)
            print(f"  {name:9s} call us " + " ".join(f"{v:7.1f}" for v in rr[:, 0]) + " | narrow kernel us "
                  + " ".join(f"{v:7.1f}" for v in rr[:, 1]) + f" | best {gb / (rr[:, 1].min() * 1e-6):7.1f} GB/s", flush=True)
        a.close()
        b.close()


if __name__ == "__main__":
    main()
