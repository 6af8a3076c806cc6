"""GPU parity of the merged K|V pool ([num_pages, page_size, Hkv, 2, D], Sec. 3.1.3
"KV merge") against the oracle's merged call: pool bit-exact, outputs within the
tolerance of the two-pool tests."""
import numpy as np
import pytest
import torch

from oracle import rpa_oracle as O
from paper_2604_15464_amd import rpa
from paper_2604_15464_amd import workloads as W

pytestmark = pytest.mark.gpu

MAX_ABS = 1.5e-2
MEAN_ABS = 2e-3


def run_merged(wl, needles=None, kv_chunk=0, narrow_waves=0, seqs=None, calls=1, causal=True, poison=True):
    dev = torch.device("cuda:0")
    if needles is None:
        x = W.materialize(wl, dev, poison=poison)
    else:
        mode, nseed = needles
        x = W.materialize_needles(wl, W.needle_targets(wl, mode, nseed, None, causal), dev, poison=poison)
    x = W.merge_pools(x)
    host = {k: W.bits(v) for k, v in x.items()}
    table_dev = torch.from_numpy(np.ascontiguousarray(wl.page_table)).to(dev)
    ctx = rpa.RaggedPagedAttention.for_workload(wl, causal=causal, kv_merged=True)
    ctx.set_options(kv_chunk=kv_chunk, narrow_waves=narrow_waves)
    out = torch.full_like(x["q"], float("nan"))
    for _ in range(calls):
        ctx.update_and_attend(x["q"], x["k_new"], x["v_new"], x["kv_pages"], None, table_dev, wl.cu_q_lens, wl.kv_lens,
                              wl.sm_scale, out=out)
    torch.cuda.synchronize()
    info = ctx.plan_info()
    ctx.close()
    ref, pool = O.update_and_attend_merged(host["q"], host["k_new"], host["v_new"], host["kv_pages"], wl.page_table,
                                           wl.cu_q_lens, wl.kv_lens, wl.num_seqs, wl.sm_scale, seqs=seqs, causal=causal)
    assert np.array_equal(W.bits(x["kv_pages"]), pool), "merged pool differs from the oracle"
    got = out.detach().to("cpu").to(torch.float64).numpy()
    rows = np.zeros(got.shape[0], dtype=bool)
    cu = wl.cu_q_lens
    for r in (range(wl.num_seqs) if seqs is None else seqs):
        rows[cu[r]:cu[r + 1]] = True
    if rows.any():
        err = np.abs(got[rows] - ref[rows])
        assert np.isfinite(got[rows]).all(), "non-finite output"
        assert err.max() <= MAX_ABS, f"max abs err {err.max():.4g}"
        assert err.mean() <= MEAN_ABS, f"mean abs err {err.mean():.4g}"
    return info


@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("needles", [None, ("spread", 2), ("random", 3)])
def test_merged_pool_ragged(seed, needles):
    """decode rows, short and long query runs, empty sequences; every batch runs narrow"""
    wl = W.ragged(1500 + seed, num_seqs=7, hq=(32, 8, 16, 8)[seed], hkv=(8, 8, 2, 1)[seed], d=128,
                  ps=(16, 64, 32, 256)[seed], max_q=(40, 3, 150, 20)[seed], max_ctx=600)
    info = run_merged(wl, needles, kv_chunk=(0, 64, 128, 32)[seed], narrow_waves=(0, 4, 2, 1)[seed])
    assert info["num_wide_units"] == 0


def test_merged_pool_repeated_calls_and_no_mask():
    wl = W.ragged(1510, num_seqs=5, hq=32, hkv=8, d=128, ps=16, max_q=30, max_ctx=300)
    run_merged(wl, calls=3)
    run_merged(wl, causal=False)


def test_merged_pool_full_size_decode():
    """config 2 at full size: N(0,1) on sampled sequences, needles on all."""
    wl = W.config(2)
    run_merged(wl, poison=False, seqs=list(range(0, wl.num_seqs, 16)))
    run_merged(wl, needles=("spread", 1), poison=False)


def test_merged_pool_rejects_what_it_has_no_kernel_for():
    with pytest.raises(rpa.RpaError):
        rpa.RaggedPagedAttention(8, 2, 64, 16, 16, 2, 4, 8, kv_merged=True)            # head_dim 64
    with pytest.raises(rpa.RpaError):
        rpa.RaggedPagedAttention(8, 2, 128, 16, 16, 2, 4, 8, kv_merged=True, kv_scales=(1.0, 1.0))   # 8-bit cache
