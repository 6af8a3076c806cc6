"""Board power beside the time per call, load by load: is a block of the benchmark
bound by what the kernel issues or by what the board may draw?

    python -m paper_2604_15464_amd.power_probe [--seconds 3]

Each load runs back to back for some seconds while a thread reads the board's power
sensor (hwmon `power1_input` / `power1_average` of the first card, microwatts) every
50 ms: MFMAs alone (`rpa_mfma_probe`), the prefill batch (config 3) on its N(0,1)
inputs, the same batch on all-zero inputs (same instructions, same addresses, hardly
a bit toggling), the decode batch (config 2) and the mixed batch (config 4).  Not part of the paper's method.
"""
import argparse
import glob
import threading
import time

import torch

from . import rpa
from . import workloads as W


def _sensor():
    for pat in ("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input",
                "/sys/class/drm/card*/device/hwmon/hwmon*/power1_average"):
        for p in sorted(glob.glob(pat)):
            try:
                with open(p) as f:
                    int(f.read())
                return p
            except (OSError, ValueError):
                continue
    return None


class _Sampler(threading.Thread):
    def __init__(self, path, period):
        super().__init__(daemon=True)
        self.path, self.period = path, period
        self.phase, self.samples, self.stop = None, {}, False

    def run(self):
        while not self.stop:
            ph = self.phase
            if ph is not None:
                try:
                    with open(self.path) as f:
                        self.samples.setdefault(ph, []).append(int(f.read()) / 1e6)
                except (OSError, ValueError):
                    pass
            time.sleep(self.period)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--seconds", type=float, default=3.0, help="length of each load")
    ap.add_argument("--gap", type=float, default=1.0, help="idle time between loads")
    args = ap.parse_args()
    path = _sensor()
    if path is None:
        raise SystemExit("power_probe: no readable hwmon power sensor")
    dev = torch.device("cuda:0")
    sampler = _Sampler(path, 0.05)
    sampler.start()

    def attend(ctx, wl, x, table, out):
        return lambda: ctx.update_and_attend(x["q"], x["k_new"], x["v_new"], x["k_pages"], x["v_pages"], table,
                                             wl.cu_q_lens, wl.kv_lens, wl.sm_scale, out=out)

    wl3, wl2 = W.config(3), W.config(2)
    x3, x2 = W.materialize(wl3, dev, poison=False), W.materialize(wl2, dev, poison=False)
    z3 = {k: (torch.zeros_like(v) if torch.is_tensor(v) and v.dtype == torch.bfloat16 else v) for k, v in x3.items()}
    t3, t2 = torch.from_numpy(wl3.page_table).to(dev), torch.from_numpy(wl2.page_table).to(dev)
    c3, c2 = rpa.RaggedPagedAttention.for_workload(wl3), rpa.RaggedPagedAttention.for_workload(wl2)
    o3, o2 = torch.empty_like(x3["q"]), torch.empty_like(x2["q"])
    wl4 = W.config(4)
    x4, t4 = W.materialize(wl4, dev, poison=False), torch.from_numpy(wl4.page_table).to(dev)
    c4, o4 = rpa.RaggedPagedAttention.for_workload(wl4), torch.empty_like(x4["q"])
    probe_steps = 2000
    probe_flops = c3.mfma_probe(probe_steps)[1]
    loads = [
        ("idle", None, None),
        ("MFMAs alone, pseudo-random operands", lambda: c3.mfma_probe(probe_steps), probe_flops),
        ("prefill 8 x 2048, N(0,1) inputs", attend(c3, wl3, x3, t3, o3), wl3.algorithmic_flops()),
        ("prefill 8 x 2048, all-zero inputs", attend(c3, wl3, z3, t3, o3), wl3.algorithmic_flops()),
        ("decode 256 x U[512,4096], N(0,1) inputs", attend(c2, wl2, x2, t2, o2), None),
        ("mixed 128 decode + 4 chunks, N(0,1) inputs", attend(c4, wl4, x4, t4, o4), None),
    ]
    cap = None
    try:
        with open(path.rsplit("/", 1)[0] + "/power1_cap") as f:
            cap = int(f.read()) / 1e6
    except (OSError, ValueError):
        pass
    print(f"sensor {path}; power cap {'%.0f W' % cap if cap else 'not readable'}; each load {args.seconds:.1f} s back to "
          f"back, {args.gap:.1f} s idle before it")
    print(f"{'load':42s} {'calls':>6s} {'us/call':>9s} {'TFLOP/s':>8s} {'W mean':>7s} {'W max':>6s} {'W last third':>12s}")
    for name, fn, flops in loads:
        torch.cuda.synchronize()
        time.sleep(args.gap)
        sampler.phase = name
        t0, n = time.perf_counter(), 0
        if fn is None:
            time.sleep(args.seconds)
        else:
            while time.perf_counter() - t0 < args.seconds:
                fn()
                n += 1
                if n % 8 == 0:
                    torch.cuda.synchronize()
            torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        sampler.phase = None
        w = sampler.samples.get(name, [0.0])
        tail = w[len(w) * 2 // 3:] or w
        us = dt / n * 1e6 if n else 0.0
        tf = f"{flops / (dt / n) / 1e12:8.1f}" if (flops and n) else f"{'':8s}"
        print(f"{name:42s} {n:6d} {us:9.1f} {tf} {sum(w) / len(w):7.0f} {max(w):6.0f} {sum(tail) / len(tail):12.0f}", flush=True)
    sampler.stop = True
    sampler.join()
    c3.close()
    c2.close()
    c4.close()


if __name__ == "__main__":
    main()
