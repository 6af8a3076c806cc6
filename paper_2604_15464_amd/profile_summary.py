"""Turn rocprofv3 output of a bench.py run into the short text / JSON summaries
kept under profiles/.

    python -m paper_2604_15464_amd.profile_summary kernels <dir-or-db> <out.txt> "<command>"
        rocprofv3 --kernel-trace --stats (rocpd database): per-kernel call count,
        total and average duration, launch shape of this library's kernels.

    python -m paper_2604_15464_amd.profile_summary traffic <fetch-dir> <write-dir> <out.json> <out.txt> "<command>"
        two rocprofv3 --pmc runs with --output-format csv (FETCH_SIZE, then
        WRITE_SIZE; both count KiB per dispatch): HBM bytes per launch of each
        of this library's kernels, each counter scaled by what it reads for the
        plain copy kernel (rpa_copy_kernel) of known size that
        `bench.py --copy-bytes` runs in the same process.

    python -m paper_2604_15464_amd.profile_summary counters <pmc-dir> <out.txt> "<command>"
        any other rocprofv3 --pmc run (csv): steady-state mean of every counter
        for each of this library's kernels.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import sqlite3
import sys

KERNELS = ("rpa_narrow_kernel", "rpa_wide_kernel", "rpa_mixed_kernel", "rpa_combine_kernel", "rpa_copy_kernel", "rpa_mfma_kernel",
           "rpa_quantize_kernel")


def short_name(name: str) -> str:
    for k in KERNELS:
        if k in name:
            tail = name.split(k, 1)[1]
            targs = tail.split(">", 1)[0] + ">" if tail.startswith("<") else ""
            return k + targs
    return name if len(name) <= 60 else name[:57] + "..."


def find(path: str, pattern: str) -> str:
    if os.path.isfile(path):
        return path
    hits = sorted(glob.glob(os.path.join(path, "**", pattern), recursive=True))
    if not hits:
        raise SystemExit(f"no {pattern} under {path}")
    return hits[-1]


def kernels(src: str, out: str, command: str) -> None:
    cur = sqlite3.connect(find(src, "*.db")).cursor()
    lines = [f"command: {command}", "source: rocprofv3 --kernel-trace --stats (rocpd database, view top_kernels)", "",
             f"{'kernel':44s} {'calls':>6s} {'total_us':>12s} {'avg_us':>10s} {'pct':>6s}"]
    for name, calls, total, avg, pct in cur.execute(
            "select name,total_calls,total_duration,average,percentage from top_kernels"):
        lines.append(f"{short_name(name):44s} {calls:6d} {total:12.1f} {avg:10.2f} {pct:6.2f}")
    rows = [r for r in cur.execute("select name,start,end,grid_x,grid_y,workgroup_x,lds_size,vgpr_count,"
                                   "accum_vgpr_count,scratch_size from kernels order by start")
            if any(k in r[0] for k in KERNELS)]
    # bench.py runs its blocks one after the other, with input generation and a context
    # set-up in between: launches of one kernel that lie less than 5 ms apart form one
    # burst, i.e. belong to one block of the bench line.  Per kernel and burst (in the order
    # bench.py runs its blocks): the average over the second half of the launches (steady
    # state, after warm-up), the launch shape, and the first launches in order (how long
    # the kernel takes while the clocks settle).
    by = collections.defaultdict(list)
    for r in rows:
        name = short_name(r[0])
        if not by[name] or r[1] - by[name][-1][-1][2] > 5e6:
            by[name].append([])
        by[name][-1].append(r)
    lines += ["", "this library's kernels, per burst of launches (= per block of the bench line that launches the kernel, "
              "in the order bench.py runs its blocks): steady average (last half of the burst) and launch shape"]
    for name, groups in by.items():
        for gi, rs in enumerate(groups):
            tail = rs[len(rs) // 2:]
            avg = sum(r[2] - r[1] for r in tail) / len(tail) / 1e3
            r = rs[-1]
            lines.append(f"  {name:40s} burst {gi + 1} n={len(rs):4d} steady_avg_us={avg:9.2f} grid_threads=({r[3]},{r[4]}) "
                         f"wg={r[5]} lds={r[6]} vgpr={r[7]} agpr={r[8]} scratch={r[9]}")
            if len(rs) >= 8:
                lines.append("    first launches (us): " + " ".join(f"{(q[2] - q[1]) / 1e3:.1f}" for q in rs[:25]))
    text = "\n".join(lines) + "\n"
    with open(out, "w") as f:
        f.write(text)
    print(text)


def read_counter(path: str, counter: str) -> dict:
    """kernel (without template arguments) -> per-dispatch (value, grid size) of
    `counter`, in dispatch order."""
    vals = collections.defaultdict(list)
    with open(find(path, "*counter_collection.csv"), newline="") as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] != counter:
                continue
            name = r["Kernel_Name"]
            if not any(k in name for k in KERNELS):
                continue
            base = next(k for k in KERNELS if k in name)
            vals[base].append((int(r["Dispatch_Id"]), float(r["Counter_Value"]), int(r["Grid_Size"])))
    return {k: [(v, g) for _, v, g in sorted(rows)] for k, rows in vals.items()}


def traffic(fetch_dir: str, write_dir: str, out_json: str, out_txt: str, command: str) -> None:
    with open(find(fetch_dir, "bench*.json")) as f:
        bench = json.loads(f.read().strip().splitlines()[-1])
    copy_bytes = int(bench["stream_copy"]["bytes"])
    fetch = read_counter(fetch_dir, "FETCH_SIZE")
    write = read_counter(write_dir, "WRITE_SIZE")

    def steady(rows):
        tail = rows[len(rows) // 2:]
        return sum(v for v, _ in tail) / len(tail)

    kib = 1024.0
    cf = copy_bytes / (steady(fetch["rpa_copy_kernel"]) * kib)
    cw = copy_bytes / (steady(write["rpa_copy_kernel"]) * kib)
    # Which kernels a block of the bench line launches.  A run must be made so that
    # every dispatch of a kernel belongs to one block (bench.py --only / --no-decode);
    # "call" adds up all kernels of a block that launches several.
    blocks = []
    if bench.get("value") is not None:
        blocks.append((bench["config"], ("rpa_narrow_kernel",)))
    if "prefill" in bench:
        blocks.append((bench["prefill"]["config"], ("rpa_wide_kernel",)))
    if "mixed" in bench:
        # one launch with both kinds of workgroup, or (other shapes) the two kernels
        blocks.append((bench["mixed"]["config"], ("rpa_mixed_kernel", "rpa_narrow_kernel", "rpa_wide_kernel",
                                                  "rpa_combine_kernel")))
    if "long_decode" in bench:
        blocks.append((bench["long_decode"]["config"], ("rpa_narrow_kernel",)))
    used = collections.Counter(k for _, ks in blocks for k in ks if k != "rpa_combine_kernel")
    if any(n > 1 for n in used.values()):
        raise SystemExit(f"a kernel is launched by several blocks of this run ({dict(used)}): profile them apart")
    try:
        with open(out_json) as f:
            out = json.load(f)
    except Exception:
        out = {}
    out.setdefault("runs", {})
    lines = [f"command: {command}",
             "source: two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch), csv output",
             f"calibration: rpa_copy_kernel moves {copy_bytes} B each way; FETCH_SIZE reads "
             f"{steady(fetch['rpa_copy_kernel']):.0f} KiB -> scale {cf:.4f}; WRITE_SIZE reads "
             f"{steady(write['rpa_copy_kernel']):.0f} KiB -> scale {cw:.4f}", "",
             f"{'workload':28s} {'kernel':20s} {'fetch_B':>14s} {'write_B':>14s} {'hbm_B/launch':>14s} "
             f"{'algorithmic_B':>14s} {'ratio':>6s}"]
    for cfg, ks in blocks:
        wname, alg = cfg["name"], cfg["algorithmic_bytes_per_step"]
        out[wname] = {}
        out["runs"][wname] = {"command": command, "calibration": {"copy_bytes": copy_bytes, "fetch_scale": cf,
                                                                   "write_scale": cw}}
        tot_f = tot_w = 0.0
        for kname in ks:
            if kname not in fetch:
                continue
            fb = steady(fetch[kname]) * kib * cf
            wb = steady(write[kname]) * kib * cw
            tot_f += fb
            tot_w += wb
            out[wname][kname] = {"hbm_bytes_per_launch": round(fb + wb), "fetch_bytes": round(fb),
                                 "write_bytes": round(wb), "launches": len(fetch[kname]),
                                 "grids": dict(collections.Counter(g for _, g in fetch[kname]))}
            if len(ks) == 1:
                out[wname][kname]["algorithmic_bytes"] = alg
            lines.append(f"{wname:28s} {kname:20s} {fb:14.0f} {wb:14.0f} {fb + wb:14.0f} "
                         + (f"{alg:14d} {(fb + wb) / alg:6.3f}" if len(ks) == 1 else ""))
        if len(ks) > 1:
            out[wname]["call"] = {"hbm_bytes_per_launch": round(tot_f + tot_w), "fetch_bytes": round(tot_f),
                                  "write_bytes": round(tot_w), "algorithmic_bytes": alg}
            lines.append(f"{wname:28s} {'call (all kernels)':20s} {tot_f:14.0f} {tot_w:14.0f} {tot_f + tot_w:14.0f} "
                         f"{alg:14d} {(tot_f + tot_w) / alg:6.3f}")
    with open(out_json, "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    text = "\n".join(lines) + "\n"
    with open(out_txt, "w") as f:
        f.write(text)
    print(text)


def counters(src: str, out: str, command: str) -> None:
    vals = collections.defaultdict(lambda: collections.defaultdict(list))
    with open(find(src, "*counter_collection.csv"), newline="") as f:
        for r in csv.DictReader(f):
            name = r["Kernel_Name"]
            if any(k in name for k in KERNELS):
                vals[short_name(name)][r["Counter_Name"]].append((int(r["Dispatch_Id"]), float(r["Counter_Value"])))
    lines = [f"command: {command}", "source: rocprofv3 --pmc, csv output; mean over the last half of each kernel's dispatches", ""]
    for kname, cs in vals.items():
        lines.append(kname)
        for cname in sorted(cs):
            rows = [v for _, v in sorted(cs[cname])]
            tail = rows[len(rows) // 2:]
            lines.append(f"  {cname:36s} n={len(rows):3d} mean={sum(tail) / len(tail):18.1f}")
    text = "\n".join(lines) + "\n"
    with open(out, "w") as f:
        f.write(text)
    print(text)


def main(argv):
    if len(argv) >= 5 and argv[1] == "kernels":
        kernels(argv[2], argv[3], argv[4])
    elif len(argv) >= 5 and argv[1] == "counters":
        counters(argv[2], argv[3], argv[4])
    elif len(argv) >= 7 and argv[1] == "traffic":
        traffic(argv[2], argv[3], argv[4], argv[5], argv[6])
    else:
        raise SystemExit(__doc__)


if __name__ == "__main__":
    main(sys.argv)
