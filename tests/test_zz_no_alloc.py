"""rpa_update_and_attend_noalloc (no context, no allocation in the library; the
work list and the split partials live in a static device array) against
rpa_update_and_attend on the same inputs, and both against the CPU oracle:
cache bit for bit, outputs within the path's tolerance.  Two calls in a row on
one GPU, the second with a smaller batch, so that what the first call left in
the array must not matter."""
import numpy as np
import pytest
import torch

from oracle import rpa_oracle as O
from paper_2604_15464_amd import rpa
from paper_2604_15464_amd import workloads as W

pytestmark = pytest.mark.gpu

MAX_ABS = 1.5e-2
MEAN_ABS = 2e-3


def _run_both(wl, seqs=None):
    dev = torch.device("cuda:0")
    x = W.materialize(wl, dev, poison=True)
    host = {k: W.bits(v) for k, v in x.items()}
    table = torch.from_numpy(wl.page_table).to(dev)
    # the existing entry point, on copies of the pools
    kp1, vp1 = x["k_pages"].clone(), x["v_pages"].clone()
    ctx = rpa.RaggedPagedAttention.for_workload(wl)
    out1 = torch.full_like(x["q"], float("nan"))
    ctx.update_and_attend(x["q"], x["k_new"], x["v_new"], kp1, vp1, table, wl.cu_q_lens, wl.kv_lens, wl.sm_scale,
                          out=out1)
    torch.cuda.synchronize()
    info = ctx.plan_info()
    shape = ctx.shape
    ctx.close()
    # the entry point that allocates nothing
    kp2, vp2 = x["k_pages"].clone(), x["v_pages"].clone()
    out2 = torch.full_like(x["q"], float("nan"))
    st = torch.cuda.current_stream(dev)
    rpa.update_and_attend_noalloc(shape, 0, out2.data_ptr(), x["q"].data_ptr(), x["k_new"].data_ptr(),
                                  x["v_new"].data_ptr(), kp2.data_ptr(), vp2.data_ptr(), table.data_ptr(),
                                  wl.cu_q_lens, wl.kv_lens, wl.sm_scale, st.cuda_stream)
    torch.cuda.synchronize()
    ref, kp_ref, vp_ref = O.update_and_attend(host["q"], host["k_new"], host["v_new"], host["k_pages"],
                                              host["v_pages"], wl.page_table, wl.cu_q_lens, wl.kv_lens,
                                              wl.num_seqs, wl.sm_scale, seqs=seqs)
    t = wl.num_tokens
    rows = np.zeros(t, dtype=bool)      # the rows the oracle computed: all, or those of `seqs`
    for r in (range(wl.num_seqs) if seqs is None else seqs):
        rows[wl.cu_q_lens[r]:wl.cu_q_lens[r + 1]] = True
    assert np.array_equal(W.bits(kp2), W.bits(kp1)) and np.array_equal(W.bits(vp2), W.bits(vp1))
    assert np.array_equal(W.bits(kp2), kp_ref) and np.array_equal(W.bits(vp2), vp_ref)
    a = out1[:t].to("cpu").to(torch.float64).numpy()
    b = out2[:t].to("cpu").to(torch.float64).numpy()
    assert np.isfinite(b).all()
    for got in (a, b):
        err = np.abs(got - ref[:t])[rows]
        assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, (err.max(), err.mean())
    d = np.abs(a - b)
    assert d.max() <= MAX_ABS and d.mean() <= MEAN_ABS
    return info


def test_noalloc_matches_context_entry_point_twice_in_a_row():
    # a mixed batch with KV splits (partials and a combine pass go through the array) ...
    big = W.ragged(4100, num_seqs=40, hq=32, hkv=8, d=128, ps=16, max_q=300, max_ctx=3000, p_decode=0.6)
    info = _run_both(big)
    assert info["max_splits"] > 1 and info["num_wide_units"] > 0 and info["num_narrow_units"] > 0
    # ... then a smaller one, whose work list and partials cover only part of what the first left behind
    small = W.config(1)
    _run_both(small)
    # and a decode batch with other head counts, page size and head_dim
    _run_both(W.ragged(4101, num_seqs=9, hq=8, hkv=2, d=256, ps=64, max_q=1, max_ctx=2500, p_decode=1.0, p_empty=0.0))


def test_noalloc_large_mixed_batch():
    """128 decode sequences and 4 chunks of 512 tokens: large enough that both entry
    points put narrow and wide workgroups into one launch.  The oracle attends a sample
    of the sequences (both kinds); the two entry points are compared on every row."""
    wl = W.config(4)
    long = [int(r) for r in np.flatnonzero(wl.q_lens > 1)]
    short = [int(r) for r in np.flatnonzero(wl.q_lens == 1)]
    info = _run_both(wl, seqs=long[:2] + short[:3] + short[-2:])
    assert info["concurrent"] == 2


def test_noalloc_rejects_what_does_not_fit():
    wl = W.config(1)
    dev = torch.device("cuda:0")
    x = W.materialize(wl, dev, poison=False)
    table = torch.from_numpy(wl.page_table).to(dev)
    before = x["k_pages"].clone()
    out = torch.full_like(x["q"], float("nan"))
    keep = out.clone()
    st = torch.cuda.current_stream(dev).cuda_stream

    def call(shape, cu, kv, scale=wl.sm_scale):
        rpa.update_and_attend_noalloc(shape, 0, out.data_ptr(), x["q"].data_ptr(), x["k_new"].data_ptr(),
                                      x["v_new"].data_ptr(), x["k_pages"].data_ptr(), x["v_pages"].data_ptr(),
                                      table.data_ptr(), cu, kv, scale, st)

    shape = rpa.make_shape(wl.num_q_heads, wl.num_kv_heads, wl.head_dim, wl.page_size, wl.num_tokens, wl.num_seqs,
                           wl.max_pages_per_seq, wl.num_pages)
    with pytest.raises(rpa.RpaError) as e:      # the 8-bit cache has no room for its staging copy here
        call(rpa.make_shape(wl.num_q_heads, wl.num_kv_heads, wl.head_dim, wl.page_size, wl.num_tokens, wl.num_seqs,
                            wl.max_pages_per_seq, wl.num_pages, kv_scales=(1.0, 1.0)), wl.cu_q_lens, wl.kv_lens)
    assert e.value.code == rpa.ERR_UNSUPPORTED
    bad = wl.kv_lens.copy()
    bad[2] = 3
    with pytest.raises(rpa.RpaError) as e:
        call(shape, wl.cu_q_lens, bad)
    assert e.value.code == rpa.ERR_BAD_LENGTHS
    with pytest.raises(rpa.RpaError) as e:
        call(shape, wl.cu_q_lens, wl.kv_lens, scale=0.0)
    assert e.value.code == rpa.ERR_INVALID_ARG
    # a batch whose work list exceeds the 64 KiB the array holds for it: 3000 one-token sequences
    n = 3000
    many = rpa.make_shape(32, 8, 128, 16, n, n, 4, 64)
    with pytest.raises(rpa.RpaError) as e:
        rpa.update_and_attend_noalloc(many, 0, 16, 16, 16, 16, 16, 16, 16, np.arange(n + 1, dtype=np.int32),
                                      np.full(n, 40, np.int32), 0.1, st)   # pointers are never dereferenced
    assert e.value.code == rpa.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.equal(before.view(torch.int16), x["k_pages"].view(torch.int16))
    assert torch.equal(out.view(torch.int16), keep.view(torch.int16))
