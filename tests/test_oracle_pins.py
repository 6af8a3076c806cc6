"""Pins of the CPU oracle against things other than itself (CPU only).

Each test is chosen so that a plausible mistake in oracle/rpa_oracle.py (a
wrong mask offset, a transposed operand, a wrong GQA map, a wrong page slot, a
dropped normalisation) fails at least one of them.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import rpa_oracle as O
from paper_2604_15464_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def host_inputs(wl, poison=True, max_tokens=None):
    t = W.materialize(wl, "cpu", poison=poison, max_tokens=max_tokens)
    return {k: W.bits(v) for k, v in t.items()}


def run_oracle(wl, x, **kw):
    return O.update_and_attend(x["q"], x["k_new"], x["v_new"], x["k_pages"], x["v_pages"],
                               wl.page_table, wl.cu_q_lens, wl.kv_lens, wl.num_seqs,
                               wl.sm_scale, **kw)


def f32_to_bf16_bits(a):
    return O.f64_to_bf16(np.asarray(a, dtype=np.float64))


def contiguous_kv(wl, x, r):
    """K/V of sequence r as contiguous fp64, built without the oracle's
    gather: cached part straight from the pool, new part from k_new."""
    ps = wl.page_size
    ctx = int(wl.ctx_lens[r])
    q0 = int(wl.cu_q_lens[r])
    lq = int(wl.q_lens[r])
    ks, vs = [], []
    for pos in range(ctx):
        pg = wl.page_table[r, pos // ps]
        ks.append(x["k_pages"][pg, pos % ps])
        vs.append(x["v_pages"][pg, pos % ps])
    for t in range(lq):
        ks.append(x["k_new"][q0 + t])
        vs.append(x["v_new"][q0 + t])
    k = O.bf16_to_f64(np.stack(ks))
    v = O.bf16_to_f64(np.stack(vs))
    q = O.bf16_to_f64(x["q"][q0:q0 + lq])
    return q, k, v


# ---- bf16 decode ----------------------------------------------------------
def test_bf16_decode_matches_torch():
    bits = np.arange(0, 65536, dtype=np.uint32).astype(np.uint16)
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    got = O.bf16_to_f64(bits)
    both_nan = np.isnan(ref) & np.isnan(got)
    assert np.array_equal(ref[~both_nan], got[~both_nan])
    assert np.array_equal(np.isnan(ref), np.isnan(got))


def test_bf16_encode_matches_torch():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))
    ref = torch.from_numpy(x).to(torch.float32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(O.f64_to_bf16(x), ref)


# ---- P1: brute force on contiguous KV --------------------------------------
@pytest.mark.parametrize("case", ["config1", "ragged7", "ragged8"])
def test_bruteforce_matches(case):
    if case == "config1":
        wl = W.config(1)
    else:
        wl = W.ragged(int(case[-1]), num_seqs=4, hq=4, hkv=2, d=8, ps=16, max_q=9, max_ctx=21)
    x = host_inputs(wl)
    out, _, _ = run_oracle(wl, x)
    for r in range(wl.num_seqs):
        lq = int(wl.q_lens[r])
        if lq == 0:
            continue
        q, k, v = contiguous_kv(wl, x, r)
        if case == "config1":
            # keep the pure-Python loop short: the two decode rows and a
            # few rows of the longer sequences
            rows = sorted({0, lq // 2, lq - 1})
        else:
            rows = range(lq)
        q0 = int(wl.cu_q_lens[r])
        ctx = int(wl.ctx_lens[r])
        for i in rows:
            ref = O.dense_bruteforce(q[i:i + 1].tolist(), k[:ctx + i + 1].tolist(),
                                     v[:ctx + i + 1].tolist(), wl.sm_scale)
            assert np.allclose(out[q0 + i], np.asarray(ref[0]), rtol=0, atol=1e-12)


def test_gqa_head_map():
    """Make KV heads very different so that a wrong head->group map shows."""
    wl = W.ragged(3, num_seqs=2, hq=6, hkv=3, d=8, ps=16, max_q=5, max_ctx=9, p_empty=0.0)
    x = host_inputs(wl)
    # V of kv head g is the constant g+1 everywhere (cached and new)
    for g in range(3):
        c = f32_to_bf16_bits(np.full(8, g + 1.0))
        x["v_pages"][:, :, g, :] = c
        x["v_new"][:, g, :] = c
    out, _, _ = run_oracle(wl, x)
    t = wl.num_tokens
    for h in range(6):
        assert np.allclose(out[:t, h, :], h // 2 + 1.0, atol=1e-12)


# ---- P2: page permutation invariance ---------------------------------------
def test_page_permutation_invariance():
    wl = W.ragged(11, num_seqs=6, max_q=30, max_ctx=70)
    x = host_inputs(wl)
    out, kp, vp = run_oracle(wl, x)
    rng = np.random.default_rng(5)
    perm = rng.permutation(wl.num_pages)          # old page id -> new page id
    x2 = dict(x)
    x2["k_pages"] = np.empty_like(x["k_pages"])
    x2["v_pages"] = np.empty_like(x["v_pages"])
    x2["k_pages"][perm] = x["k_pages"]
    x2["v_pages"][perm] = x["v_pages"]
    table2 = np.where(wl.page_table >= 0, perm[np.maximum(wl.page_table, 0)], -1).astype(np.int32)
    out2, kp2, vp2 = O.update_and_attend(x2["q"], x2["k_new"], x2["v_new"], x2["k_pages"],
                                         x2["v_pages"], table2, wl.cu_q_lens, wl.kv_lens,
                                         wl.num_seqs, wl.sm_scale)
    t = wl.num_tokens
    assert np.array_equal(out[:t], out2[:t])
    assert np.array_equal(kp2[perm], kp)
    assert np.array_equal(vp2[perm], vp)


# ---- P3: decode equals the last row of the matching prefill ---------------
def test_decode_equals_last_prefill_row():
    hq, hkv, d, ps = 4, 2, 16, 16
    c = 37
    rng = np.random.default_rng(21)
    tok_q = f32_to_bf16_bits(rng.standard_normal((c + 1, hq, d)))
    tok_k = f32_to_bf16_bits(rng.standard_normal((c + 1, hkv, d)))
    tok_v = f32_to_bf16_bits(rng.standard_normal((c + 1, hkv, d)))
    # prefill of c+1 tokens into empty pages
    wl_p = W.Workload("p", 0, hq, hkv, d, ps, 8, [c + 1], [c + 1],
                      W.make_page_table([c + 1], ps, 8, np.random.default_rng(1)))
    pool = np.full((8, ps, hkv, d), W.POISON_BITS, dtype=np.uint16)
    out_p, kp, vp = O.update_and_attend(tok_q, tok_k, tok_v, pool, pool.copy(), wl_p.page_table,
                                        wl_p.cu_q_lens, wl_p.kv_lens, 1, wl_p.sm_scale)
    # decode: first c tokens already cached (through a different page table)
    wl_d = W.Workload("d", 0, hq, hkv, d, ps, 8, [1], [c + 1],
                      W.make_page_table([c + 1], ps, 8, np.random.default_rng(2)))
    kpool = np.full((8, ps, hkv, d), W.POISON_BITS, dtype=np.uint16)
    vpool = kpool.copy()
    for pos in range(c):
        pg = wl_d.page_table[0, pos // ps]
        kpool[pg, pos % ps] = tok_k[pos]
        vpool[pg, pos % ps] = tok_v[pos]
    out_d, _, _ = O.update_and_attend(tok_q[c:], tok_k[c:], tok_v[c:], kpool, vpool,
                                      wl_d.page_table, wl_d.cu_q_lens, wl_d.kv_lens, 1,
                                      wl_d.sm_scale)
    assert np.allclose(out_d[0], out_p[c], rtol=0, atol=1e-13)


# ---- P4: chunk composition across calls -------------------------------------
def test_chunked_prefill_composition():
    hq, hkv, d, ps = 4, 2, 16, 16
    total, chunk = 80, 20
    rng = np.random.default_rng(33)
    tq = f32_to_bf16_bits(rng.standard_normal((total, hq, d)))
    tk = f32_to_bf16_bits(rng.standard_normal((total, hkv, d)))
    tv = f32_to_bf16_bits(rng.standard_normal((total, hkv, d)))
    table = W.make_page_table([total], ps, 7, np.random.default_rng(3))
    empty = np.full((7, ps, hkv, d), W.POISON_BITS, dtype=np.uint16)
    scale = float(np.float32(0.25))
    out_full, kp_full, vp_full = O.update_and_attend(
        tq, tk, tv, empty, empty.copy(), table, np.array([0, total], np.int32),
        np.array([total], np.int32), 1, scale)
    kp, vp = empty.copy(), empty.copy()
    outs = []
    for c0 in range(0, total, chunk):
        o, kp, vp = O.update_and_attend(
            tq[c0:c0 + chunk], tk[c0:c0 + chunk], tv[c0:c0 + chunk], kp, vp, table,
            np.array([0, chunk], np.int32), np.array([c0 + chunk], np.int32), 1, scale)
        outs.append(o)
    assert np.array_equal(kp, kp_full) and np.array_equal(vp, vp_full)
    assert np.allclose(np.concatenate(outs), out_full, rtol=0, atol=1e-12)


# ---- P5: library special case ----------------------------------------------
@pytest.mark.parametrize("d", [32, 256])
@pytest.mark.parametrize("lq,ctx", [(1, 40), (33, 0), (17, 29)])
def test_matches_torch_sdpa_float64(lq, ctx, d):
    hq, hkv, ps = 8, 2, 16
    wl = W.Workload("s", 9, hq, hkv, d, ps, 6, [lq], [lq + ctx],
                    W.make_page_table([lq + ctx], ps, 6, np.random.default_rng(4)))
    x = host_inputs(wl)
    out, _, _ = run_oracle(wl, x)
    q, k, v = contiguous_kv(wl, x, 0)
    tq = torch.from_numpy(q).permute(1, 0, 2)                       # [Hq, lq, D]
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(hq // hkv, dim=0)
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(hq // hkv, dim=0)
    i = torch.arange(lq)[:, None]
    j = torch.arange(lq + ctx)[None, :]
    mask = j <= (ctx + i)
    ref = torch.nn.functional.scaled_dot_product_attention(
        tq[None], tk[None], tv[None], attn_mask=mask, scale=wl.sm_scale)[0]
    assert np.allclose(out[:lq], ref.permute(1, 0, 2).numpy(), rtol=0, atol=1e-12)


# ---- P6: closed forms ------------------------------------------------------
def test_golden_uniform_mean():
    spec = {}
    with open(os.path.join(GOLDEN, "uniform_mean.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *vals = line.split()
            spec[key] = [float(v) for v in vals]
    ctx, lq = int(spec["ctx"][0]), int(spec["q_len"][0])
    d, ps = 4, 16
    vals = np.asarray(spec["v"])
    q = np.zeros((lq, 1, d), dtype=np.uint16)
    k_new = f32_to_bf16_bits(np.random.default_rng(0).standard_normal((lq, 1, d)))
    v_new = f32_to_bf16_bits(np.repeat(vals[ctx:, None, None], d, axis=2))
    kp = np.full((2, ps, 1, d), W.POISON_BITS, dtype=np.uint16)
    vp = kp.copy()
    kp[1, :ctx] = f32_to_bf16_bits(np.random.default_rng(1).standard_normal((ctx, 1, d)))
    vp[1, :ctx] = f32_to_bf16_bits(np.repeat(vals[:ctx, None, None], d, axis=2))
    out, _, _ = O.update_and_attend(q, k_new, v_new, kp, vp, np.array([[1]], np.int32),
                                    np.array([0, lq], np.int32), np.array([ctx + lq], np.int32),
                                    1, 0.5)
    for i, e in enumerate(spec["expect"]):
        assert np.allclose(out[i, 0], e, atol=1e-14)


def test_constant_v_gives_constant():
    wl = W.ragged(12, num_seqs=5, max_q=20, max_ctx=50)
    x = host_inputs(wl)
    const = f32_to_bf16_bits(np.linspace(-2, 2, wl.head_dim))
    x["v_pages"][:] = const
    x["v_new"][:] = const
    out, _, _ = run_oracle(wl, x)
    t = wl.num_tokens
    assert np.allclose(out[:t], O.bf16_to_f64(const), atol=1e-13)


def test_equal_keys_give_prefix_mean():
    hq, hkv, d, ps = 2, 1, 8, 16
    lq, ctx = 6, 11
    wl = W.Workload("e", 13, hq, hkv, d, ps, 4, [lq], [lq + ctx],
                    W.make_page_table([lq + ctx], ps, 4, np.random.default_rng(6)))
    x = host_inputs(wl)
    row = f32_to_bf16_bits(np.random.default_rng(7).standard_normal(d))
    x["k_pages"][:] = row
    x["k_new"][:] = row
    out, _, _ = run_oracle(wl, x)
    _, _, v = contiguous_kv(wl, x, 0)
    for i in range(lq):
        assert np.allclose(out[i, 0], v[:ctx + i + 1, 0].mean(axis=0), atol=1e-13)
        assert np.allclose(out[i, 1], v[:ctx + i + 1, 0].mean(axis=0), atol=1e-13)


def test_single_token_returns_v_new():
    wl = W.Workload("one", 14, 4, 2, 16, 16, 2, [1], [1],
                    W.make_page_table([1], 16, 2, np.random.default_rng(8)))
    x = host_inputs(wl)
    out, _, _ = run_oracle(wl, x)
    v = O.bf16_to_f64(x["v_new"][0])
    for h in range(4):
        assert np.array_equal(out[0, h], v[h // 2])


def test_two_keys_logistic():
    """Softmax over two keys is the logistic function of the score gap."""
    d, ps = 4, 16
    q = f32_to_bf16_bits(np.array([[[1.0, 0.0, 0.0, 0.0]]]))
    k0, k1 = 0.75, -1.5                 # bf16-exact
    kp = np.zeros((1, ps, 1, d), dtype=np.uint16)
    vp = np.zeros((1, ps, 1, d), dtype=np.uint16)
    kp[0, 0] = f32_to_bf16_bits([k0, 3, 3, 3])
    vp[0, 0] = f32_to_bf16_bits([1.0, 0.0, 2.0, -4.0])
    k_new = f32_to_bf16_bits(np.array([[[k1, -7, 5, 1]]]))
    v_new = f32_to_bf16_bits(np.array([[[0.0, 1.0, -2.0, 4.0]]]))
    scale = 0.5
    out, _, _ = O.update_and_attend(q, k_new, v_new, kp, vp, np.array([[0]], np.int32),
                                    np.array([0, 1], np.int32), np.array([2], np.int32), 1, scale)
    gap = scale * (k0 - k1)
    w0 = 0.5 * (1.0 + math.tanh(gap / 2.0))
    expect = w0 * np.array([1.0, 0.0, 2.0, -4.0]) + (1 - w0) * np.array([0.0, 1.0, -2.0, 4.0])
    assert np.allclose(out[0, 0], expect, atol=1e-14)


def test_key_shift_invariance():
    """Adding the same vector to every key adds a per-query constant to all
    its scores, which softmax ignores."""
    hq, hkv, d, ps = 2, 2, 8, 16
    lq, ctx = 5, 9
    wl = W.Workload("sh", 15, hq, hkv, d, ps, 3, [lq], [lq + ctx],
                    W.make_page_table([lq + ctx], ps, 3, np.random.default_rng(9)))
    x = host_inputs(wl, poison=False)
    # small integers: sums stay exact in bf16
    rng = np.random.default_rng(10)
    for name in ("k_pages", "k_new"):
        x[name] = f32_to_bf16_bits(rng.integers(-3, 4, size=x[name].shape).astype(np.float64))
    out, _, _ = run_oracle(wl, x)
    shift = rng.integers(-2, 3, size=d).astype(np.float64)
    x2 = dict(x)
    for name in ("k_pages", "k_new"):
        x2[name] = f32_to_bf16_bits(O.bf16_to_f64(x[name]) + shift)
    out2, _, _ = run_oracle(wl, x2)
    assert np.allclose(out[:lq], out2[:lq], atol=1e-12)


# ---- P7: split-merge identity ----------------------------------------------
def test_split_merge_identity():
    rng = np.random.default_rng(41)
    d, n = 16, 77
    q = rng.standard_normal(d)
    k = rng.standard_normal((n, d)) * 3
    v = rng.standard_normal((n, d))
    scale = 0.3
    full = O.attend_sequence(q[None, None, :], k[:, None, :], v[:, None, :], np.float32(scale))[0, 0]
    scale32 = float(np.float32(scale))
    for cuts in ([0, 77], [0, 10, 77], [0, 1, 2, 50, 50, 77], [0, 16, 32, 48, 64, 77]):
        parts = [O.partial_attention(q, k[a:b], v[a:b], scale32) for a, b in zip(cuts[:-1], cuts[1:])]
        assert np.allclose(O.merge_partials(parts), full, atol=1e-13)


# ---- P8: sentinel bytes / poison -------------------------------------------
def test_only_new_slots_change_and_poison_is_ignored():
    wl = W.ragged(17, num_seqs=6, max_q=25, max_ctx=60, spare_pages=4)
    x = host_inputs(wl, poison=True, max_tokens=wl.num_tokens + 3)
    out, kp, vp = run_oracle(wl, x)
    t = wl.num_tokens
    assert np.isfinite(out[:t]).all()
    assert np.isnan(out[t:]).all()
    # slots that must have changed: exactly the new positions
    changed = np.zeros((wl.num_pages, wl.page_size), dtype=bool)
    for r in range(wl.num_seqs):
        for pos in range(int(wl.ctx_lens[r]), int(wl.kv_lens[r])):
            changed[wl.page_table[r, pos // wl.page_size], pos % wl.page_size] = True
    assert changed.sum() == t
    assert np.array_equal(kp[~changed], x["k_pages"][~changed])
    assert np.array_equal(vp[~changed], x["v_pages"][~changed])
    # and they hold the new rows, bit for bit
    for r in range(wl.num_seqs):
        q0 = int(wl.cu_q_lens[r])
        for i in range(int(wl.q_lens[r])):
            pos = int(wl.ctx_lens[r]) + i
            pg, sl = wl.page_table[r, pos // wl.page_size], pos % wl.page_size
            assert np.array_equal(kp[pg, sl], x["k_new"][q0 + i])
            assert np.array_equal(vp[pg, sl], x["v_new"][q0 + i])
    # inputs untouched
    x_again = host_inputs(wl, poison=True, max_tokens=wl.num_tokens + 3)
    assert np.array_equal(x["k_pages"], x_again["k_pages"])


# ---- P9: idempotence -------------------------------------------------------
def test_idempotent_on_updated_cache():
    wl = W.ragged(19, num_seqs=5, max_q=25, max_ctx=60)
    x = host_inputs(wl)
    out, kp, vp = run_oracle(wl, x)
    x2 = dict(x, k_pages=kp, v_pages=vp)
    out2, kp2, vp2 = run_oracle(wl, x2)
    t = wl.num_tokens
    assert np.array_equal(out[:t], out2[:t])
    assert np.array_equal(kp, kp2) and np.array_equal(vp, vp2)


# ---- mask offset: a planted off-by-one must be visible ----------------------
def test_mask_extent_is_inclusive_of_own_token():
    """Query i must see its own token (position ctx+i) and nothing later:
    make the own token's V huge and the next token's V different."""
    d, ps = 4, 16
    lq, ctx = 3, 2
    q = np.zeros((lq, 1, d), dtype=np.uint16)
    k_new = np.zeros((lq, 1, d), dtype=np.uint16)
    vals = np.array([0.0, 0.0, 8.0, 16.0, 32.0])          # positions 0..4
    v_new = f32_to_bf16_bits(np.repeat(vals[ctx:, None, None], d, axis=2))
    kp = np.zeros((1, ps, 1, d), dtype=np.uint16)
    vp = np.zeros((1, ps, 1, d), dtype=np.uint16)
    out, _, _ = O.update_and_attend(q, k_new, v_new, kp, vp, np.array([[0]], np.int32),
                                    np.array([0, lq], np.int32), np.array([ctx + lq], np.int32),
                                    1, 1.0)
    assert np.allclose(out[:, 0, 0], [8.0 / 3, 24.0 / 4, 56.0 / 5], atol=1e-14)


def test_config_shapes():
    """The generators give what the workload list states."""
    c1 = W.config(1)
    assert c1.q_lens.tolist() == [1, 1, 50, 20] and c1.kv_lens.tolist() == [37, 90, 50, 70]
    assert (c1.num_q_heads, c1.num_kv_heads, c1.head_dim, c1.page_size, c1.num_pages) == (4, 2, 64, 16, 64)
    c2 = W.config(2)
    assert c2.num_seqs == 256 and c2.kv_lens.min() >= 512 and c2.kv_lens.max() <= 4096
    assert (c2.q_lens == 1).all()
    c3 = W.config(3)
    assert c3.q_lens.tolist() == [2048] * 8 and c3.kv_lens.tolist() == [2048] * 8
    assert c3.algorithmic_flops() == 4 * 32 * 128 * 8 * (2048 * 2049 // 2)
    c4 = W.config(4)
    assert c4.num_seqs == 132 and c4.num_tokens == 128 + 4 * 512
    assert sorted((c4.kv_lens - c4.q_lens)[c4.q_lens == 512].tolist()) == [1024, 2048, 4096, 8192]
    c5 = W.config(5)
    assert c5.num_seqs == 32 and c5.page_size == 64
    assert c5.kv_lens.min() >= 32768 and c5.kv_lens.max() <= 131072
    for c in (c1, c2, c3, c4, c5):
        used = c.page_table[c.page_table >= 0]
        assert len(np.unique(used)) == len(used)
        assert used.max() < c.num_pages


# ---- non-causal reading (causal=False: every query sees all kv_len positions) ----
def test_noncausal_bruteforce_matches():
    wl = W.ragged(21, num_seqs=4, hq=4, hkv=2, d=8, ps=16, max_q=9, max_ctx=21)
    x = host_inputs(wl)
    out, kp, vp = run_oracle(wl, x, causal=False)
    out_c, kp_c, vp_c = run_oracle(wl, x)
    # the mask does not change what is written into the cache
    assert np.array_equal(kp, kp_c) and np.array_equal(vp, vp_c)
    for r in range(wl.num_seqs):
        lq = int(wl.q_lens[r])
        if lq == 0:
            continue
        q, k, v = contiguous_kv(wl, x, r)
        q0 = int(wl.cu_q_lens[r])
        for i in range(lq):
            # the brute force sees the whole sequence for every row ...
            ref = O.dense_bruteforce(q[i:i + 1].tolist(), k.tolist(), v.tolist(), wl.sm_scale, causal=False)
            assert np.allclose(out[q0 + i], np.asarray(ref[0]), rtol=0, atol=1e-12)
        # ... and the last row sees the same keys under either mask
        assert np.allclose(out[q0 + lq - 1], out_c[q0 + lq - 1], rtol=0, atol=1e-13)


@pytest.mark.parametrize("lq,ctx", [(1, 40), (33, 0), (17, 29)])
def test_noncausal_matches_torch_sdpa_float64(lq, ctx):
    hq, hkv, d, ps = 8, 2, 32, 16
    wl = W.Workload("s", 9, hq, hkv, d, ps, 6, [lq], [lq + ctx],
                    W.make_page_table([lq + ctx], ps, 6, np.random.default_rng(4)))
    x = host_inputs(wl)
    out, _, _ = run_oracle(wl, x, causal=False)
    q, k, v = contiguous_kv(wl, x, 0)
    tq = torch.from_numpy(q).permute(1, 0, 2)
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(hq // hkv, dim=0)
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(hq // hkv, dim=0)
    ref = torch.nn.functional.scaled_dot_product_attention(tq[None], tk[None], tv[None], scale=wl.sm_scale)[0]
    assert np.allclose(out[:lq], ref.permute(1, 0, 2).numpy(), rtol=0, atol=1e-12)


def test_noncausal_closed_forms():
    hq, hkv, d, ps = 2, 1, 8, 16
    lq, ctx = 6, 11
    wl = W.Workload("e", 13, hq, hkv, d, ps, 4, [lq], [lq + ctx],
                    W.make_page_table([lq + ctx], ps, 4, np.random.default_rng(6)))
    x = host_inputs(wl)
    # equal keys: every row is the mean of ALL values, later tokens included
    row = f32_to_bf16_bits(np.random.default_rng(7).standard_normal(d))
    x["k_pages"][:] = row
    x["k_new"][:] = row
    out, _, _ = run_oracle(wl, x, causal=False)
    _, _, v = contiguous_kv(wl, x, 0)
    for i in range(lq):
        assert np.allclose(out[i, 0], v[:, 0].mean(axis=0), atol=1e-13)
    # equal queries: rows of one head are identical (nothing depends on the row index)
    x = host_inputs(wl)
    x["q"][:lq] = x["q"][0]
    out, _, _ = run_oracle(wl, x, causal=False)
    for i in range(1, lq):
        assert np.allclose(out[i], out[0], atol=1e-13)
    # while under the causal mask they differ (later rows see more keys)
    out_c, _, _ = run_oracle(wl, x)
    assert not np.allclose(out_c[0], out_c[lq - 1], atol=1e-6)


# ---- 8-bit KV cache (E4M3 bytes, one scale per tensor) --------------------------------------
KV_SCALES = (1.0 / 64.0, 1.0 / 32.0)


def run_oracle_fp8(wl, x, scales=KV_SCALES, **kw):
    return O.update_and_attend(x["q"], x["k_new"], x["v_new"], x["k_pages"], x["v_pages"],
                               wl.page_table, wl.cu_q_lens, wl.kv_lens, wl.num_seqs,
                               wl.sm_scale, kv_scales=scales, **kw)


def host_inputs_fp8(wl, scales=KV_SCALES, poison=True):
    t = W.materialize(wl, "cpu", poison=poison, kv_scales=scales)
    return {k: W.bits(v) for k, v in t.items()}


def test_e4m3_decode_matches_torch_and_format():
    b = np.arange(256, dtype=np.uint8)
    ref = torch.from_numpy(b.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = O.e4m3_to_f64(b)
    assert np.array_equal(np.isnan(got), np.isnan(ref)) and np.isnan(got).sum() == 2
    assert np.array_equal(got[~np.isnan(got)], ref[~np.isnan(ref)])
    # the format's fixed points: bias 7, largest value 448, smallest 2**-9
    assert got[0x38] == 1.0 and got[0x7E] == 448.0 and got[0x01] == 2.0 ** -9 and got[0x08] == 2.0 ** -6
    assert got[0x80] == 0.0 and np.signbit(got[0x80]) and got[0xFE] == -448.0


def test_e4m3_encode_matches_torch_and_nearest_search():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.normal(size=20000) * 3, rng.normal(size=20000) * 150, rng.normal(size=5000) * 1e-2,
                        rng.normal(size=2000) * 1e-3]).astype(np.float32)
    x = np.clip(x, -448, 448)
    got = O.f32_to_e4m3(x)
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(got, ref)
    # structurally different: nearest of the 254 finite values, ties to the even code
    table = O.e4m3_to_f64(np.arange(256, dtype=np.uint8))
    for v, code in zip(x[::97].tolist(), got[::97].tolist()):
        dist = np.abs(table - v)
        dist[np.isnan(dist)] = np.inf
        best = np.flatnonzero(dist == dist.min())
        if v == 0.0 or abs(table[code]) == 0.0:
            assert table[code] == 0.0 and 0 in (best & 0x7F)
            continue
        cands = [c for c in best if np.signbit(table[c]) == np.signbit(v)]
        assert code in cands
        if len(cands) == 2:                        # a tie: the even mantissa wins
            assert code % 2 == 0


def test_e4m3_encode_special_cases():
    enc = lambda *v: O.f32_to_e4m3(np.asarray(v, dtype=np.float32)).tolist()
    assert enc(0.0, 1.0, -1.0) == [0x00, 0x38, 0xB8]
    assert enc(1.0625, 1.1875) == [0x38, 0x3A]                 # ties go to the even mantissa
    assert enc(448.0, 449.0, 464.0, 465.0, 1e6, np.inf) == [0x7E] * 6     # saturates, never a NaN byte
    assert enc(-500.0, -np.inf) == [0xFE, 0xFE]
    assert enc(2.0 ** -9, 2.0 ** -10, 1.5 * 2.0 ** -9, 2.0 ** -6) == [0x01, 0x00, 0x02, 0x08]
    # every finite byte survives a round trip
    b = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    assert np.array_equal(O.f32_to_e4m3(O.e4m3_to_f64(b).astype(np.float32)), b)
    # half an ulp of three mantissa bits in the normal range
    x = np.random.default_rng(3).uniform(2.0 ** -6, 448, size=5000).astype(np.float32)
    err = np.abs(O.e4m3_to_f64(O.f32_to_e4m3(x)) - x) / x
    assert err.max() <= 2.0 ** -4


def test_fp8_cache_update_writes_quantised_rows_only():
    wl = W.ragged(7, num_seqs=5, hq=4, hkv=2, d=16, ps=16, max_q=20, max_ctx=50)
    x = host_inputs_fp8(wl)
    _, kp, vp = run_oracle_fp8(wl, x)
    assert kp.dtype == np.uint8
    changed = np.zeros(kp.shape[:2], dtype=bool)
    for r in range(wl.num_seqs):
        q0, lq, ctx = int(wl.cu_q_lens[r]), int(wl.q_lens[r]), int(wl.ctx_lens[r])
        for t in range(lq):
            pos = ctx + t
            pg = wl.page_table[r, pos // wl.page_size]
            changed[pg, pos % wl.page_size] = True
            for name, pool, scale in (("k_new", kp, KV_SCALES[0]), ("v_new", vp, KV_SCALES[1])):
                val = O.bf16_to_f64(x[name][q0 + t]).astype(np.float32) * (np.float32(1) / np.float32(scale))
                ref = torch.from_numpy(np.clip(val, -448, 448)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
                assert np.array_equal(pool[pg, pos % wl.page_size], ref)
    assert np.array_equal(kp[~changed], x["k_pages"][~changed]) and np.array_equal(vp[~changed], x["v_pages"][~changed])


def test_fp8_path_equals_bf16_path_on_dequantised_inputs():
    """Attention over the 8-bit cache is plain attention over value(byte) * scale: feed
    those values (exact in bf16 for power-of-two scales) to the 16-bit path."""
    wl = W.ragged(8, num_seqs=5, hq=4, hkv=2, d=16, ps=16, max_q=20, max_ctx=50)
    x = host_inputs_fp8(wl, poison=False)
    out8, kp8, vp8 = run_oracle_fp8(wl, x)
    y = dict(x)
    y["k_pages"] = f32_to_bf16_bits(O.e4m3_to_f64(x["k_pages"]) * KV_SCALES[0])
    y["v_pages"] = f32_to_bf16_bits(O.e4m3_to_f64(x["v_pages"]) * KV_SCALES[1])
    y["k_new"] = f32_to_bf16_bits(O.e4m3_to_f64(O.quantize_rows(x["k_new"], KV_SCALES[0])) * KV_SCALES[0])
    y["v_new"] = f32_to_bf16_bits(O.e4m3_to_f64(O.quantize_rows(x["v_new"], KV_SCALES[1])) * KV_SCALES[1])
    out16, _, _ = run_oracle(wl, y)
    live = ~np.isnan(out16)
    assert np.array_equal(np.isnan(out8), np.isnan(out16))
    assert np.allclose(out8[live], out16[live], rtol=0, atol=1e-12)


def test_fp8_power_of_two_scale_invariance():
    """Doubling the new rows and both scales leaves the stored bytes unchanged; the
    bytes then stand for doubled K and V, so with half the softmax scale the output
    is exactly doubled (away from the subnormal and saturation ends of the format)."""
    wl = W.ragged(9, num_seqs=4, hq=4, hkv=2, d=16, ps=16, max_q=12, max_ctx=0)      # new tokens only
    xa = host_inputs_fp8(wl)
    xb = dict(xa)
    xb["k_new"] = f32_to_bf16_bits(O.bf16_to_f64(xa["k_new"]) * 2.0)
    xb["v_new"] = f32_to_bf16_bits(O.bf16_to_f64(xa["v_new"]) * 2.0)
    oa, ka, va = run_oracle_fp8(wl, xa)
    ob, kb, vb = O.update_and_attend(xb["q"], xb["k_new"], xb["v_new"], xb["k_pages"], xb["v_pages"], wl.page_table,
                                     wl.cu_q_lens, wl.kv_lens, wl.num_seqs, wl.sm_scale / 2,
                                     kv_scales=(2 * KV_SCALES[0], 2 * KV_SCALES[1]))
    assert np.array_equal(ka, kb) and np.array_equal(va, vb)
    live = ~np.isnan(oa)
    assert live.any() and np.allclose(2.0 * oa[live], ob[live], rtol=0, atol=1e-12)


def test_fp8_decode_equals_last_prefill_row():
    """q_len 1 on a cache that an earlier call filled == last row of the one-call prefill."""
    hq, hkv, d, ps, n = 4, 2, 16, 16, 23
    rng = np.random.default_rng(11)
    wl_full = W.Workload("f", 3, hq, hkv, d, ps, 4, [n], [n], W.make_page_table([n], ps, 4, rng))
    x = host_inputs_fp8(wl_full)
    out_full, kp, vp = run_oracle_fp8(wl_full, x)
    wl_pre = W.Workload("p", 3, hq, hkv, d, ps, 4, [n - 1], [n - 1], wl_full.page_table)
    _, kp1, vp1 = run_oracle_fp8(wl_pre, x)
    wl_dec = W.Workload("d", 3, hq, hkv, d, ps, 4, [1], [n], wl_full.page_table)
    y = dict(x)
    y["k_pages"], y["v_pages"] = kp1, vp1
    for name in ("q", "k_new", "v_new"):
        y[name] = x[name][n - 1:n]
    out_dec, kp2, vp2 = run_oracle_fp8(wl_dec, y)
    assert np.array_equal(kp2, kp) and np.array_equal(vp2, vp)
    assert np.allclose(out_dec[0], out_full[n - 1], rtol=0, atol=1e-12)


# ---- merged K|V pool (Sec. 3.1.3 "KV merge") -------------------------------------
def test_merged_pool_bruteforce_and_equals_two_pool_call():
    """The pool is filled here token by token from contiguous K/V lists (not by
    the packing helper), attention is checked against the pure-Python brute
    force, and the whole call against the two-pool oracle on the same data."""
    wl = W.ragged(5, num_seqs=4, hq=4, hkv=2, d=8, ps=16, max_q=9, max_ctx=37, p_empty=0.0)
    x = host_inputs(wl)
    ps = wl.page_size
    pool = np.full((wl.num_pages, ps, wl.num_kv_heads, 2, wl.head_dim), W.POISON_BITS, dtype=np.uint16)
    for r in range(wl.num_seqs):
        for pos in range(int(wl.ctx_lens[r])):
            pg = wl.page_table[r, pos // ps]
            for g in range(wl.num_kv_heads):
                pool[pg, pos % ps, g, 0] = x["k_pages"][pg, pos % ps, g]
                pool[pg, pos % ps, g, 1] = x["v_pages"][pg, pos % ps, g]
    out_m, pool_after = O.update_and_attend_merged(x["q"], x["k_new"], x["v_new"], pool, wl.page_table, wl.cu_q_lens,
                                                   wl.kv_lens, wl.num_seqs, wl.sm_scale)
    for r in range(wl.num_seqs):
        q, k, v = contiguous_kv(wl, x, r)
        q0, ctx = int(wl.cu_q_lens[r]), int(wl.ctx_lens[r])
        for i in range(int(wl.q_lens[r])):
            ref = O.dense_bruteforce(q[i:i + 1].tolist(), k[:ctx + i + 1].tolist(), v[:ctx + i + 1].tolist(), wl.sm_scale)
            assert np.allclose(out_m[q0 + i], np.asarray(ref[0]), rtol=0, atol=1e-12)
    out_s, k_after, v_after = run_oracle(wl, x)
    t = wl.num_tokens
    assert np.array_equal(out_m[:t], out_s[:t])
    out_mn, _ = O.update_and_attend_merged(x["q"], x["k_new"], x["v_new"], pool, wl.page_table, wl.cu_q_lens,
                                           wl.kv_lens, wl.num_seqs, wl.sm_scale, causal=False)
    assert np.array_equal(out_mn[:t], run_oracle(wl, x, causal=False)[0][:t]) and not np.array_equal(out_mn[:t], out_m[:t])
    live_or_new = (pool_after[:, :, :, 0, :] != W.POISON_BITS).all(axis=(2, 3))
    assert np.array_equal(pool_after[live_or_new][:, :, 0], k_after[live_or_new])
    assert np.array_equal(pool_after[live_or_new][:, :, 1], v_after[live_or_new])
    # exactly the pre-existing slots and this call's slots hold data
    written = np.zeros_like(live_or_new)
    for r in range(wl.num_seqs):
        for pos in range(int(wl.kv_lens[r])):
            written[wl.page_table[r, pos // ps], pos % ps] = True
    assert np.array_equal(live_or_new, written)
    assert (pool_after[~written] == W.POISON_BITS).all()


def test_merged_pool_k_and_v_are_not_swapped():
    """V constant per (half): if the pool's two halves were read the other way
    round the output would be the keys' constant."""
    wl = W.ragged(6, num_seqs=3, hq=4, hkv=2, d=8, ps=16, max_q=4, max_ctx=20, p_empty=0.0)
    x = host_inputs(wl, poison=False)
    x["v_pages"][:] = f32_to_bf16_bits(np.full(8, 3.0))
    x["v_new"][:] = f32_to_bf16_bits(np.full(8, 3.0))
    m = W.merge_pools(x)
    assert m["kv_pages"].shape == (wl.num_pages, wl.page_size, 2, 2, 8)
    out, pool = O.update_and_attend_merged(m["q"], m["k_new"], m["v_new"], m["kv_pages"], wl.page_table, wl.cu_q_lens,
                                           wl.kv_lens, wl.num_seqs, wl.sm_scale)
    assert np.allclose(out[:wl.num_tokens], 3.0, atol=1e-12)
    r = 0
    pos = int(wl.kv_lens[r]) - 1
    pg = wl.page_table[r, pos // 16]
    last_tok = int(wl.cu_q_lens[r + 1]) - 1
    assert np.array_equal(pool[pg, pos % 16, :, 0], x["k_new"][last_tok])
    assert np.array_equal(pool[pg, pos % 16, :, 1], x["v_new"][last_tok])
