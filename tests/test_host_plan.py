"""CPU tests of the C-ABI library's host side: it loads, exports what the header
declares, validates lengths, and its work partition covers every (query token,
KV position) pair exactly once with exactly one cache writer per token."""
import os
import re

import numpy as np
import pytest

from paper_2604_15464_amd import rpa
from paper_2604_15464_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
F = {n: i for i, n in enumerate(rpa.UNIT_FIELDS)}


def shape_of(wl, max_tokens=None, max_seqs=None, causal=True, kv_scales=None):
    return rpa.make_shape(wl.num_q_heads, wl.num_kv_heads, wl.head_dim, wl.page_size,
                          max_tokens or max(1, wl.num_tokens), max_seqs or max(1, wl.num_seqs),
                          wl.max_pages_per_seq, wl.num_pages, causal, kv_scales)


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "rpa.h")) as f:
        text = f.read()
    declared = set(re.findall(r"^(?:int|void|const char\*)\s+(rpa_\w+)\s*\(", text, flags=re.M))
    assert declared == set(rpa.EXPORTS)
    l = rpa.lib()
    for name in declared:
        assert hasattr(l, name), name


def check_plan(wl, units, items, stats, narrow_tq, wide_tq=None, causal=True):
    wide_tq = wide_tq or stats["wide_rows"] // (wl.num_q_heads // wl.num_kv_heads)
    cu = wl.cu_q_lens
    # per token: covered KV positions and writers
    cover = {}
    writers = np.zeros(wl.num_tokens, dtype=np.int64)
    tile_units = {}
    for u in units:
        seq, q_start, q_pos0, n_q = u[F["seq"]], u[F["q_start"]], u[F["q_pos0"]], u[F["n_q"]]
        b, e, ctx, seq_q0, part, flags = (u[F["kv_begin"]], u[F["kv_end"]], u[F["ctx"]], u[F["seq_q0"]],
                                          u[F["part_row"]], u[F["flags"]])
        wide = bool(flags & 2)
        assert seq_q0 == cu[seq] and q_start == seq_q0 + q_pos0
        assert ctx == wl.kv_lens[seq] - wl.q_lens[seq]
        assert 1 <= n_q <= (wide_tq if wide else narrow_tq)
        assert q_pos0 + n_q <= wl.q_lens[seq]
        assert 0 <= b < e <= (ctx + q_pos0 + n_q if causal else wl.kv_lens[seq])
        assert b % (64 if wide else 16) == 0
        tile_units.setdefault((seq, q_pos0), []).append((b, e, part, flags, n_q))
        if flags & 1:
            writers[q_start:q_start + n_q] += 1
    assert (writers == 1).all()
    n_items = 0
    for (seq, q_pos0), lst in tile_units.items():
        lst.sort()
        n_q = lst[0][4]
        kv_hi = wl.kv_lens[seq] - wl.q_lens[seq] + q_pos0 + n_q if causal else wl.kv_lens[seq]
        # ranges tile [0, kv_hi) without gap or overlap
        assert lst[0][0] == 0 and lst[-1][1] == kv_hi
        for (b0, e0, *_), (b1, *_rest) in zip(lst[:-1], lst[1:]):
            assert e0 == b1
        if len(lst) == 1:
            assert lst[0][2] == -1
        else:
            n_items += 1
            rows = n_q * wl.num_q_heads
            parts = [p for _, _, p, _, _ in lst]
            assert all(p >= 0 for p in parts)
            assert [p - parts[0] for p in parts] == [i * rows for i in range(len(lst))]
            match = [it for it in items if it[0] == parts[0]]
            assert len(match) == 1
            assert match[0].tolist() == [parts[0], len(lst), rows, cu[seq] + q_pos0]
    assert n_items == len(items) == stats["num_combine_items"]
    # every query token appears in exactly one tile
    seen = np.zeros(wl.num_tokens, dtype=np.int64)
    for (seq, q_pos0), lst in tile_units.items():
        seen[cu[seq] + q_pos0: cu[seq] + q_pos0 + lst[0][4]] += 1
    assert (seen == 1).all()
    # partial rows do not overlap
    spans = sorted((it[0], it[0] + it[1] * it[2]) for it in items)
    for (a0, a1), (b0, b1) in zip(spans[:-1], spans[1:]):
        assert a1 <= b0
    if spans:
        assert spans[-1][1] == stats["partial_rows"]


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("variant", [rpa.VARIANT_AUTO, rpa.VARIANT_DECODE, rpa.VARIANT_PREFILL, rpa.VARIANT_MIXED])
def test_plan_covers_configs(idx, variant):
    wl = W.config(idx) if idx in (1, 2, 5) else W.config(idx, scale=0.25)
    units, items, stats = rpa.plan_host(shape_of(wl), wl.cu_q_lens, wl.kv_lens, variant=variant)
    check_plan(wl, units, items, stats, narrow_tq=16 // (wl.num_q_heads // wl.num_kv_heads))
    if variant == rpa.VARIANT_DECODE:
        assert stats["num_wide_units"] == 0 and stats["variant"] == rpa.VARIANT_DECODE
    if variant == rpa.VARIANT_PREFILL:
        assert stats["num_narrow_units"] == 0 and stats["variant"] == rpa.VARIANT_PREFILL


@pytest.mark.parametrize("idx", [1, 3, 4])
@pytest.mark.parametrize("variant", [rpa.VARIANT_AUTO, rpa.VARIANT_DECODE, rpa.VARIANT_PREFILL])
def test_plan_without_causal_mask_covers_whole_sequences(idx, variant):
    wl = W.config(idx) if idx == 1 else W.config(idx, scale=0.25)
    units, items, stats = rpa.plan_host(shape_of(wl, causal=False), wl.cu_q_lens, wl.kv_lens, variant=variant,
                                        kv_chunk=64, wide_kv_chunk=64)
    check_plan(wl, units, items, stats, narrow_tq=16 // (wl.num_q_heads // wl.num_kv_heads), causal=False)


@pytest.mark.parametrize("variant", [rpa.VARIANT_AUTO, rpa.VARIANT_DECODE, rpa.VARIANT_PREFILL])
def test_plan_head_dim_256(variant):
    """head_dim 256: 128-row wide tiles only, at most four waves per narrow
    workgroup (LDS), and the options that ask for more are rejected."""
    wl = W.ragged(1200, num_seqs=9, hq=32, hkv=8, d=256, ps=16, max_q=150, max_ctx=400)
    units, items, stats = rpa.plan_host(shape_of(wl), wl.cu_q_lens, wl.kv_lens, variant=variant, num_cus=256)
    check_plan(wl, units, items, stats, narrow_tq=4)
    assert stats["wide_rows"] == 128 and stats["narrow_waves"] == 4
    big = W.uniform(8, 4096, 4096, d=256)          # enough tiles for the 256-row shape at head_dim 128
    assert rpa.plan_host(shape_of(big), big.cu_q_lens, big.kv_lens, num_cus=256)[2]["wide_rows"] == 128
    for kw in ({"wide_rows": 256}, {"narrow_waves": 8}):
        with pytest.raises(rpa.RpaError) as e:
            rpa.plan_host(shape_of(wl), wl.cu_q_lens, wl.kv_lens, **kw)
        assert e.value.code == rpa.ERR_INVALID_ARG


def test_mixed_batches_run_side_by_side_when_large_enough():
    c4 = W.config(4)
    assert rpa.plan_host(shape_of(c4), c4.cu_q_lens, c4.kv_lens)[2]["concurrent"] == 1
    assert rpa.plan_host(shape_of(c4), c4.cu_q_lens, c4.kv_lens, mixed_overlap=1)[2]["concurrent"] == 0
    c1 = W.config(1)                                  # tiny, but one launch can hold both parts: side by side
    assert rpa.plan_host(shape_of(c1), c1.cu_q_lens, c1.kv_lens)[2]["concurrent"] == 1
    assert rpa.plan_host(shape_of(c1), c1.cu_q_lens, c1.kv_lens, mixed_overlap=1)[2]["concurrent"] == 0
    # where that launch is not built (head_dim 256) a tiny batch is not worth two stream packets
    t256 = W.ragged(77, num_seqs=6, hq=8, hkv=2, d=256, ps=16, max_q=60, max_ctx=200, p_decode=0.5)
    assert (t256.q_lens == 1).any() and (t256.q_lens > 8).any()
    assert rpa.plan_host(shape_of(t256), t256.cu_q_lens, t256.kv_lens)[2]["concurrent"] == 0
    assert rpa.plan_host(shape_of(t256), t256.cu_q_lens, t256.kv_lens, mixed_overlap=2)[2]["concurrent"] == 1
    for idx in (2, 3):                                # one kind of work only: nothing to overlap
        wl = W.config(idx, scale=0.25)
        assert rpa.plan_host(shape_of(wl), wl.cu_q_lens, wl.kv_lens, mixed_overlap=2)[2]["concurrent"] == 0
    # 3 = side by side as two kernels on two streams, whatever the sizes
    assert rpa.plan_host(shape_of(c1), c1.cu_q_lens, c1.kv_lens, mixed_overlap=3)[2]["concurrent"] == 1
    with pytest.raises(rpa.RpaError):
        rpa.plan_host(shape_of(c1), c1.cu_q_lens, c1.kv_lens, mixed_overlap=4)


def test_plan_with_8bit_cache():
    """The 8-bit cache has a wide kernel at head_dim 128 only (elsewhere every tile is
    narrow, whatever variant is asked for), keeps eight narrow waves per CU unless a
    wide workgroup is to run beside them, and refuses unusable scales."""
    sc = (1 / 64, 1 / 32)
    for d in (64, 256):
        wl = W.ragged(1700 + d, num_seqs=9, hq=8, hkv=2, d=d, ps=16, max_q=150, max_ctx=400)
        for variant in (rpa.VARIANT_AUTO, rpa.VARIANT_PREFILL):
            units, items, stats = rpa.plan_host(shape_of(wl, kv_scales=sc), wl.cu_q_lens, wl.kv_lens, variant=variant)
            check_plan(wl, units, items, stats, narrow_tq=4)
            assert stats["num_wide_units"] == 0 and stats["variant"] == rpa.VARIANT_DECODE
    wl = W.ragged(1828, num_seqs=9, hq=32, hkv=8, d=128, ps=16, max_q=150, max_ctx=400)
    units, items, stats = rpa.plan_host(shape_of(wl, kv_scales=sc), wl.cu_q_lens, wl.kv_lens)
    check_plan(wl, units, items, stats, narrow_tq=4)
    assert stats["num_wide_units"] > 0
    c2, c4 = W.config(2), W.config(4)
    assert rpa.plan_host(shape_of(c2), c2.cu_q_lens, c2.kv_lens)[2]["num_narrow_bins"] == 128
    assert rpa.plan_host(shape_of(c2, kv_scales=sc), c2.cu_q_lens, c2.kv_lens)[2]["num_narrow_bins"] == 256
    s4 = rpa.plan_host(shape_of(c4, kv_scales=sc), c4.cu_q_lens, c4.kv_lens)[2]
    assert s4["concurrent"] == 1 and s4["num_narrow_bins"] == 128
    for bad in ((0.0, 1.0), (1.0, -2.0), (float("nan"), 1.0), (1.0, float("inf")), (1e-45, 1.0)):
        with pytest.raises(rpa.RpaError) as e:
            rpa.plan_host(shape_of(c2, kv_scales=bad), c2.cu_q_lens, c2.kv_lens)
        assert e.value.code == rpa.ERR_INVALID_ARG


def test_auto_variant_follows_distribution():
    s2 = rpa.plan_host(shape_of(W.config(2)), W.config(2).cu_q_lens, W.config(2).kv_lens)[2]
    assert s2["variant"] == rpa.VARIANT_DECODE
    c3 = W.config(3, scale=0.25)
    assert rpa.plan_host(shape_of(c3), c3.cu_q_lens, c3.kv_lens)[2]["variant"] == rpa.VARIANT_PREFILL
    c4 = W.config(4, scale=0.25)
    assert rpa.plan_host(shape_of(c4), c4.cu_q_lens, c4.kv_lens)[2]["variant"] == rpa.VARIANT_MIXED


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("kv_chunk", [0, 16, 48])
def test_plan_covers_random_ragged(seed, kv_chunk):
    wl = W.ragged(100 + seed, num_seqs=9, max_q=150, max_ctx=400)
    units, items, stats = rpa.plan_host(shape_of(wl), wl.cu_q_lens, wl.kv_lens, kv_chunk=kv_chunk,
                                        wide_kv_chunk=64 if kv_chunk else 0)
    check_plan(wl, units, items, stats, narrow_tq=8)
    if kv_chunk:
        assert stats["max_splits"] > 1


def test_decode_bins_balance_bytes():
    """Narrow units are dealt into bins of equal KV volume: one workgroup per bin,
    every bin within a few tiles of the mean, bins contiguous in the unit list."""
    for idx in (2, 5):
        wl = W.config(idx)
        units, _, stats = rpa.plan_host(shape_of(wl), wl.cu_q_lens, wl.kv_lens, num_cus=256)
        bins = units[:, F["bin"]]
        assert (np.diff(bins) >= 0).all() and bins[0] == 0 and bins[-1] == stats["num_narrow_bins"] - 1
        tiles = -(-(units[:, F["kv_end"]] - units[:, F["kv_begin"]]) // 16)
        per_bin = np.bincount(bins, weights=tiles)
        assert stats["num_narrow_bins"] * (wl.num_kv_heads // stats["narrow_waves"]) <= 2 * 256
        assert per_bin.max() - per_bin.mean() <= 3
        assert per_bin.min() >= 0.9 * per_bin.mean() or per_bin.argmin() == len(per_bin) - 1


def test_bad_lengths_are_rejected():
    wl = W.config(1)
    sh = shape_of(wl)
    cu, kv = wl.cu_q_lens.copy(), wl.kv_lens.copy()

    def code(cu_, kv_, shape=sh):
        with pytest.raises(rpa.RpaError) as e:
            rpa.plan_host(shape, cu_, kv_)
        return e.value.code

    bad = cu.copy(); bad[0] = 1
    assert code(bad, kv) == rpa.ERR_BAD_LENGTHS
    bad = cu.copy(); bad[2] = bad[1] - 1
    assert code(bad, kv) == rpa.ERR_BAD_LENGTHS
    badkv = kv.copy(); badkv[2] = 49                     # kv_len < q_len
    assert code(cu, badkv) == rpa.ERR_BAD_LENGTHS
    badkv = kv.copy(); badkv[1] = 16 * 6 + 1             # needs 7 pages, row holds 6
    assert code(cu, badkv) == rpa.ERR_BAD_LENGTHS
    small = shape_of(wl, max_tokens=71)
    assert code(cu, kv, small) == rpa.ERR_BAD_LENGTHS
    few = shape_of(wl, max_seqs=3)
    assert code(cu, kv, few) == rpa.ERR_BAD_LENGTHS


def test_unsupported_shapes_are_rejected():
    for kw in ({"head_dim": 96}, {"page_size": 24}, {"page_size": 8}, {"num_q_heads": 6, "num_kv_heads": 4},
               {"num_q_heads": 24, "num_kv_heads": 8}):
        args = dict(num_q_heads=4, num_kv_heads=2, head_dim=64, page_size=16, max_tokens=8, max_seqs=2,
                    max_pages_per_seq=4, num_pages=8)
        args.update(kw)
        with pytest.raises(rpa.RpaError) as e:
            rpa.plan_host(rpa.make_shape(**args), [0, 1], [1])
        assert e.value.code == rpa.ERR_UNSUPPORTED


def test_empty_batches():
    wl = W.config(1)
    units, items, stats = rpa.plan_host(shape_of(wl), [0], np.zeros(0, np.int32))
    assert len(units) == 0 and len(items) == 0
    # sequences with q_len 0 contribute nothing
    units, items, stats = rpa.plan_host(shape_of(wl), [0, 0, 3, 3], [5, 10, 7])
    assert set(units[:, F["seq"]].tolist()) == {1}


def test_default_launch_rules():
    """What the partitioner picks when no knob is set, on the cases each rule was measured
    on: tile height, unit order, cuts and the narrow / wide line."""
    def plan(wl, **kw):
        kvs = kw.pop("kv_scales", None)
        return rpa.plan_host(shape_of(wl, kv_scales=kvs), wl.cu_q_lens, wl.kv_lens, **kw)

    def seq_runs(units):
        s = units[:, F["seq"]]
        return 1 + int(np.count_nonzero(s[1:] != s[:-1]))

    # prefill 8 x 2048: 256-row tiles in the persistent launch, one sequence after the other
    units, _, st = plan(W.config(3))
    assert st["wide_rows"] == 256 and st["max_splits"] == 1 and seq_runs(units) == 8
    # the same lengths with one KV head, at head_dim 256, over the 8-bit cache: longest tile first overall
    for wl, kw in ((W.regime("prefill", hq=8, hkv=1), {}), (W.regime("prefill", d=256, ps=64), {}),
                   (W.regime("prefill"), {"kv_scales": (1 / 64, 1 / 32)})):
        units, _, st = plan(wl, **kw)
        assert seq_runs(units) > 8
        span = (units[:, F["kv_end"]] - units[:, F["kv_begin"]]).astype(np.int64) * units[:, F["n_q"]]
        assert np.all(span[1:] <= span[:-1])
    # head_dim 64 and the 8-bit cache: 128-row tiles
    assert plan(W.regime("prefill", d=64))[2]["wide_rows"] == 128
    assert plan(W.regime("prefill"), kv_scales=(1 / 64, 1 / 32))[2]["wide_rows"] == 128
    # a mixed batch: 128-row tiles and side by side, however much of it is prefill
    for wl in (W.config(4), W.config(1)):
        st = plan(wl)[2]
        assert st["variant"] == rpa.VARIANT_MIXED and st["wide_rows"] == 128 and st["concurrent"] == 1
    rng = np.random.default_rng(11)
    q = np.concatenate([np.ones(64, dtype=np.int64), np.full(8, 2048, dtype=np.int64)])
    kv = np.concatenate([np.full(64, 2049, dtype=np.int64), np.full(8, 2048, dtype=np.int64)])
    heavy = W._finish("prefill_heavy_mixed", 11, 32, 8, 128, 16, q, kv, rng)
    st = plan(heavy)[2]
    assert st["wide_rows"] == 128 and st["concurrent"] == 1
    # long items under few query tiles are cut, short ones are not
    assert plan(W.uniform(4, 256, 16384 + 256, ps=16))[2]["max_splits"] > 1
    assert plan(W.uniform(1, 512, 8192 + 512, ps=16))[2]["max_splits"] > 1
    assert plan(W.uniform(2, 512, 4096 + 512, ps=16))[2]["max_splits"] == 1
    assert plan(W.uniform(1, 2048, 2048, ps=16))[2]["max_splits"] == 1
    # long, full items with one workgroup per CU: 256-row tiles
    assert plan(W.uniform(16, 128, 8192 + 128, ps=16))[2]["wide_rows"] == 256
    assert plan(W.uniform(8, 256, 2048 + 256, ps=16))[2]["wide_rows"] == 128
    # narrow up to one narrow tile of query tokens (16 / h_g = 4 here), wide beyond
    assert plan(W.uniform(64, 4, 1024, ps=16))[2]["variant"] == rpa.VARIANT_DECODE
    assert plan(W.uniform(64, 5, 1024, ps=16))[2]["variant"] == rpa.VARIANT_PREFILL
    # the mixed recipe with two KV heads: its long chunks are cut, with eight they are not
    assert plan(W.regime("mixed", hq=16, hkv=2))[2]["max_splits"] > 1
    units, _, st = plan(W.config(4))
    wide = units[(units[:, F["flags"]] & 2) != 0]
    assert np.all(wide[:, F["part_row"]] < 0)


def test_only_tile_of_a_sequence_is_flagged():
    """Bit 2 of a wide unit's flags: the unit's tile is the only query tile of its sequence,
    so no other tile of the call reads the same K/V rows (the wide kernel streams them)."""
    wl = W.ragged(4242, num_seqs=30, hq=32, hkv=8, d=128, ps=16, max_q=120, max_ctx=900, p_decode=0.3)
    units, _, st = rpa.plan_host(shape_of(wl), wl.cu_q_lens, wl.kv_lens, wide_kv_chunk=256)
    tq = {False: 16 // 4, True: st["wide_rows"] // 4}
    tiles = {}
    for u in units:
        tiles.setdefault(int(u[F["seq"]]), set()).add(int(u[F["q_pos0"]]))
    seen = set()
    for u in units:
        seq, wide = int(u[F["seq"]]), bool(u[F["flags"]] & 2)
        alone = bool(u[F["flags"]] & 4)
        if not wide:                      # the narrow kernel streams every K/V row anyway
            assert not alone
            continue
        assert alone == (len(tiles[seq]) == 1), (seq, tiles[seq])
        assert alone == (wl.q_lens[seq] <= tq[wide])
        seen.add(alone)
    assert seen == {True, False}
