"""Randomised parity run on a GPU, as long as you like (not collected by pytest):

    python tests/fuzz_gpu_parity.py SECONDS [SEED_BASE]

Draws shapes, length mixes, launch knobs, cache types and input recipes at random,
runs each batch through the C ABI and compares cache and outputs with the CPU oracle
exactly as tests/test_gpu_parity.py does.  Every case is printed before it runs, so
a failure names its seed.  (Runs of 300-840 s on different seed bases: 1900-6000 cases each,
all equal to the oracle within the tolerance.)"""
import os
import random
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import test_gpu_parity as T  # noqa: E402
from paper_2604_15464_amd import rpa, workloads as W  # noqa: E402
t_end = time.time() + float(sys.argv[1])
base = int(sys.argv[2]) if len(sys.argv) > 2 else 0
n_ok = 0; i = 0
while time.time() < t_end:
    rng = random.Random(77000 + base + i); i += 1
    hkv = rng.choice([1, 2, 4, 8]); hg = rng.choice([1, 2, 4, 8, 16])
    hq = hkv * hg if hkv * hg <= 64 else hkv * 4
    d = rng.choice([64, 128, 128, 256])
    kw = dict(variant=rng.choice([0, 0, 1, 1, 2, 3]), kv_chunk=rng.choice([0, 0, 16, 48, 160]),
              wide_kv_chunk=rng.choice([0, 0, 64, 192]), pad_tokens=rng.choice([0, 3]), pad_seqs=rng.choice([0, 2]),
              narrow_waves=rng.choice([0, 0, 1, 2]) if hkv % 2 == 0 else 0, units_per_cu=rng.choice([0, 2]),
              wide_rows=rng.choice([0, 128, 256]) if d <= 128 else 0, causal=rng.random() < 0.8,
              mixed_overlap=rng.choice([0, 1, 2, 2, 2, 3]), calls=rng.choice([1, 2]), wide_persistent=rng.choice([0, 0, 1]), upload=rng.choice([0, 0, 1, 2, 3]))
    if rng.random() < 0.3:
        kw["kv_scales"] = rng.choice([(1 / 64, 1 / 32), (0.05, 0.02), (1.0, 1.0)])
    if rng.random() < 0.5:
        kw["needles"] = (rng.choice(["boundaries", "spread", "random"]), rng.randint(0, 99))
    seqs = None
    if rng.random() < 0.04:
        # now and then a batch large enough for the launch forms that small ones never reach
        # (persistent wide workgroups, 256-row tiles by count, cut long items); the oracle
        # attends a sample of its sequences, the cache is compared in full
        wl = W.ragged(90000 + base + i, num_seqs=rng.randint(8, 40), hq=hq, hkv=hkv, d=d,
                      ps=rng.choice([16, 64, 256]), max_q=rng.choice([600, 1500, 2500]),
                      max_ctx=rng.choice([0, 2500, 9000]), p_decode=rng.choice([0.0, 0.3, 0.8]), p_empty=0.0)
        seqs = sorted(rng.sample(range(wl.num_seqs), 3))
        kw["calls"] = 1
    else:
        wl = W.ragged(90000 + base + i, num_seqs=rng.randint(1, 40), hq=hq, hkv=hkv, d=d,
                      ps=rng.choice([16, 32, 64, 128, 256]), max_q=rng.choice([1, 5, 40, 200, 500]),
                      max_ctx=rng.choice([0, 50, 700, 2500, 6000]), p_decode=rng.choice([0.1, 0.5, 0.9, 1.0]),
                      p_empty=rng.choice([0.0, 0.1]))
    if wl.num_tokens == 0: continue
    print(f"case {i}: hq{hq} hkv{hkv} d{d} ps{wl.page_size} seqs{wl.num_seqs} tok{wl.num_tokens} kvmax{int(wl.kv_lens.max())} {kw}"
          + (f" oracle on sequences {seqs}" if seqs else ""), flush=True)
    try:
        res = T.run_case(wl, seqs=seqs, **kw)
    except rpa.RpaError as e:
        assert e.code in (rpa.ERR_WORKSPACE, rpa.ERR_INVALID_ARG, rpa.ERR_UNSUPPORTED), str(e)
        print("   rejected:", e, flush=True); continue
    T.check(wl, res, seqs=seqs); n_ok += 1
print("fuzz ok:", n_ok, "cases")
