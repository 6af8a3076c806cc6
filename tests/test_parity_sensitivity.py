"""CPU only: how much the inputs of the parity tests can tell.

The oracle is run on a batch and on the same batch with a mistake planted in the
DATA the way a wrong gather would see it (two live cache slots of different
sequences swapped; a whole 16-position tile replaced by another sequence's
rows).  With N(0,1) inputs at decode lengths the outputs move by less than the
parity tolerance, i.e. such a gather mistake would pass; with the needle inputs
(workloads.materialize_needles) every targeted slot moves its output row by
O(1).  This is what entitles the GPU parity tests on needle inputs to say that
rows come from the right slots."""
import numpy as np

from oracle import rpa_oracle as O
from paper_2604_15464_amd import workloads as W

MAX_ABS = 1.5e-2


def oracle_out(wl, h, seqs=None):
    out, _, _ = O.update_and_attend(h["q"], h["k_new"], h["v_new"], h["k_pages"], h["v_pages"], wl.page_table,
                                    wl.cu_q_lens, wl.kv_lens, wl.num_seqs, wl.sm_scale, seqs=seqs)
    return out


def decode_batch():
    rng = np.random.default_rng(12)
    kv = [2300, 2300, 1500, 2301]
    return W.Workload("sens_decode", 12, 32, 8, 128, 16, 600, [1, 1, 1, 1], kv, W.make_page_table(kv, 16, 600, rng))


def swap_slots(h, wl, r_a, p_a, r_b, p_b):
    g = {k: v.copy() for k, v in h.items()}
    ps = wl.page_size
    sa, sb = int(W.slot_of_position(wl, r_a, p_a)), int(W.slot_of_position(wl, r_b, p_b))
    for name in ("k_pages", "v_pages"):
        flat = g[name].reshape(-1, wl.num_kv_heads, wl.head_dim)
        tmp = flat[sa].copy()
        flat[sa] = flat[sb]
        flat[sb] = tmp
    return g


def foreign_tile(h, wl, r_a, p0, r_b, q0):
    """positions p0..p0+15 of sequence r_a take the rows of q0..q0+15 of r_b"""
    g = {k: v.copy() for k, v in h.items()}
    for name in ("k_pages", "v_pages"):
        flat = g[name].reshape(-1, wl.num_kv_heads, wl.head_dim)
        flat[W.slot_of_position(wl, r_a, np.arange(p0, p0 + 16))] = flat[W.slot_of_position(wl, r_b, np.arange(q0, q0 + 16))]
    return g


def test_gaussian_inputs_hide_a_wrong_slot_and_needles_show_it():
    wl = decode_batch()
    # --- N(0,1): today's recipe --------------------------------------------------
    h = {k: W.bits(v) for k, v in W.materialize(wl, "cpu", poison=False).items()}
    base = oracle_out(wl, h, seqs=[0])
    moved_swap = np.abs(oracle_out(wl, swap_slots(h, wl, 0, 1000, 1, 77), seqs=[0]) - base)[0]
    moved_tile = np.abs(oracle_out(wl, foreign_tile(h, wl, 0, 1008, 1, 320), seqs=[0]) - base)[0]
    assert moved_swap.max() < MAX_ABS          # one wrong live slot: invisible
    assert moved_tile.max() < MAX_ABS          # a whole foreign tile: still under the tolerance
    # --- needles aimed at those positions -------------------------------------------
    tg = W.needle_targets(wl, "random", seed=1)
    tg[0, :] = 1000 + np.arange(32) % 16 + 8      # sequence 0: all heads inside positions 1008..1023
    tg[0, 0] = 1000
    n = {k: W.bits(v) for k, v in W.materialize_needles(wl, tg, "cpu", poison=False).items()}
    base = oracle_out(wl, n, seqs=[0])
    moved_swap = np.abs(oracle_out(wl, swap_slots(n, wl, 0, 1000, 1, 77), seqs=[0]) - base)[0]
    moved_tile = np.abs(oracle_out(wl, foreign_tile(n, wl, 0, 1008, 1, 320), seqs=[0]) - base)[0]
    assert moved_swap[0].max() > 100 * MAX_ABS          # the head aimed at the swapped slot
    assert (moved_tile[1:].max(axis=1) > 50 * MAX_ABS).all()   # every head aimed into the replaced tile


def test_spread_needles_cover_a_prefill_and_show_any_wrong_slot():
    rng = np.random.default_rng(13)
    q, kv = [400, 150], [400, 700]
    wl = W.Workload("sens_prefill", 13, 8, 2, 128, 16, 80, q, kv, W.make_page_table(kv, 16, 80, rng))
    tg = W.needle_targets(wl, "spread")
    cu = wl.cu_q_lens
    hg = wl.num_q_heads // wl.num_kv_heads
    for r in range(wl.num_seqs):
        for g in range(wl.num_kv_heads):
            seen = np.unique(tg[cu[r]:cu[r + 1], g * hg:(g + 1) * hg])
            assert len(seen) >= 0.75 * wl.kv_lens[r], (r, g, len(seen))      # most positions of every KV head are somebody's target
    n = {k: W.bits(v) for k, v in W.materialize_needles(wl, tg, "cpu", poison=False).items()}
    base = oracle_out(wl, n)
    # a cached slot of the chunked sequence that some query aims at, swapped with a slot of its neighbour page
    ctx1 = kv[1] - q[1]
    aimed = np.unique(tg[cu[1]:cu[2]])
    p = int(aimed[(aimed < ctx1) & (aimed >= 16)][5])
    g2 = {k: v.copy() for k, v in n.items()}
    for name in ("k_pages", "v_pages"):
        flat = g2[name].reshape(-1, wl.num_kv_heads, wl.head_dim)
        a, b = int(W.slot_of_position(wl, 1, p)), int(W.slot_of_position(wl, 1, p - 16))
        # K of one slot with V of the other: what a gather that mixes up two pages for one pool would see
        if name == "v_pages":
            tmp = flat[a].copy()
            flat[a] = flat[b]
            flat[b] = tmp
    moved = np.abs(oracle_out(wl, g2) - base)
    rows = np.nonzero((tg[cu[1]:cu[2]] == p).any(axis=1))[0]
    assert len(rows) > 0 and np.nanmax(moved[cu[1] + rows]) > 50 * MAX_ABS


def test_boundary_needles_sit_on_the_boundaries():
    wl = W.config(4, scale=0.0625)
    cuts = [[96, 160] if wl.kv_lens[r] > 200 else [] for r in range(wl.num_seqs)]
    tg = W.needle_targets(wl, "boundaries", cuts=cuts)
    cu = wl.cu_q_lens
    for r in range(wl.num_seqs):
        ql, kv = int(wl.q_lens[r]), int(wl.kv_lens[r])
        ctx = kv - ql
        t = tg[cu[r]:cu[r + 1]]
        assert (t <= ctx + np.arange(ql)[:, None]).all() and (t >= 0).all()      # always visible
        want = {0, kv - 1, ctx - 1 if ctx else 0} | ({95, 96, 159, 160} if cuts[r] else set())
        last_tok = set(t[-1].tolist())
        if ql * wl.num_q_heads >= 64:                 # enough queries to go round the whole list
            assert want <= set(np.unique(t).tolist()) | last_tok, (r, want - set(np.unique(t).tolist()))
