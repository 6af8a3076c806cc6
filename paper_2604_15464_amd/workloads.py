"""Seeded synthetic inputs for ragged paged attention.

This module only *describes and fills* inputs: sequence lengths, page tables
and random bf16 tensors.  It holds none of the method's arithmetic (no
attention, no cache update) so that the CPU oracle and the HIP path can both be
fed from it without sharing any code of the method itself.

The five named workloads follow the paper's evaluation shapes (Llama-3-8B
attention: 32 query heads, 8 KV heads, head_dim 128, bf16; Sec. 4 "Benchmark
Setting") but with ragged length mixes (Sec. 2.4 "Mixed Batch"): decode-only,
prefill-only and mixed batches, which are the three regimes of Sec. 3.4.
"""
from __future__ import annotations

from dataclasses import dataclass, field
import math

import numpy as np

# bf16 bit pattern used to poison cache slots that the method must never read
# or that it must overwrite: a quiet NaN.
POISON_BITS = 0x7FC1


@dataclass
class Workload:
    name: str
    seed: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    num_pages: int
    q_lens: np.ndarray            # int32 [n]
    kv_lens: np.ndarray           # int32 [n], includes this call's new tokens
    page_table: np.ndarray        # int32 [n, max_pages_per_seq], -1 = unused
    sm_scale: float = field(default=0.0)

    def __post_init__(self):
        self.q_lens = np.asarray(self.q_lens, dtype=np.int32)
        self.kv_lens = np.asarray(self.kv_lens, dtype=np.int32)
        self.page_table = np.ascontiguousarray(self.page_table, dtype=np.int32)
        if self.sm_scale == 0.0:
            self.sm_scale = float(np.float32(1.0 / math.sqrt(self.head_dim)))
        else:
            self.sm_scale = float(np.float32(self.sm_scale))

    @property
    def num_seqs(self) -> int:
        return int(self.q_lens.shape[0])

    @property
    def cu_q_lens(self) -> np.ndarray:
        cu = np.zeros(self.num_seqs + 1, dtype=np.int32)
        np.cumsum(self.q_lens, out=cu[1:])
        return cu

    @property
    def num_tokens(self) -> int:
        return int(self.q_lens.sum())

    @property
    def max_pages_per_seq(self) -> int:
        return int(self.page_table.shape[1])

    @property
    def ctx_lens(self) -> np.ndarray:
        return (self.kv_lens - self.q_lens).astype(np.int32)

    # ---- algorithmic work, used by the benchmark only -------------------
    def algorithmic_bytes(self, kv_fp8: bool = False) -> int:
        """Bytes the method itself must move (Sec. 4.1 throughput formula,
        generalised to ragged lengths): every cached or new K/V element read
        once, every new K/V element written once, q read and out written.
        With the 8-bit cache a cached element and a written one are one byte;
        the new rows still arrive as bf16."""
        d, hkv, hq = self.head_dim, self.num_kv_heads, self.num_q_heads
        kv = int(self.kv_lens.astype(np.int64).sum())
        ql = int(self.q_lens.astype(np.int64).sum())
        if kv_fp8:
            ctx = kv - ql
            return d * (2 * hkv * (ctx * 1 + ql * 2 + ql * 1) + 2 * 2 * ql * hq)
        return 2 * d * ((kv + ql) * 2 * hkv + 2 * ql * hq)

    def algorithmic_flops(self) -> int:
        """Exact causal FLOPs of the two contractions: 4*Hq*D per visible
        (query, key) pair."""
        total = 0
        for ql, kl in zip(self.q_lens.tolist(), self.kv_lens.tolist()):
            ctx = kl - ql
            total += ql * ctx + ql * (ql + 1) // 2
        return 4 * self.num_q_heads * self.head_dim * total


def pages_needed(kv_lens, page_size: int) -> np.ndarray:
    kv = np.asarray(kv_lens, dtype=np.int64)
    return ((kv + page_size - 1) // page_size).astype(np.int64)


def make_page_table(kv_lens, page_size: int, num_pages: int, rng: np.random.Generator,
                    max_pages_per_seq: int | None = None, shuffle: bool = True) -> np.ndarray:
    """Rows take consecutive slices of one permutation of the pool."""
    need = pages_needed(kv_lens, page_size)
    total = int(need.sum())
    if total > num_pages:
        raise ValueError(f"pool of {num_pages} pages too small for {total}")
    width = int(max(1, need.max() if need.size else 1))
    if max_pages_per_seq is not None:
        if max_pages_per_seq < width:
            raise ValueError("max_pages_per_seq too small")
        width = max_pages_per_seq
    perm = rng.permutation(num_pages) if shuffle else np.arange(num_pages)
    table = np.full((len(need), width), -1, dtype=np.int32)
    off = 0
    for r, n in enumerate(need.tolist()):
        table[r, :n] = perm[off:off + n]
        off += n
    return table


def _finish(name, seed, hq, hkv, d, ps, q_lens, kv_lens, rng, num_pages=None,
            max_pages_per_seq=None, shuffle=True) -> Workload:
    need = int(pages_needed(kv_lens, ps).sum())
    if num_pages is None:
        num_pages = need
    table = make_page_table(kv_lens, ps, num_pages, rng, max_pages_per_seq, shuffle)
    return Workload(name, seed, hq, hkv, d, ps, num_pages, q_lens, kv_lens, table)


def config(index: int, scale: float = 1.0) -> Workload:
    """The five evaluation workloads.  `scale` < 1 shrinks the lengths (and
    for index 2-5 the number of sequences) for CPU-sized parity cases while
    keeping the regime and the length distribution."""
    if index == 1:
        rng = np.random.default_rng(1)
        q = [1, 1, 50, 20]
        kv = [37, 90, 50, 70]
        return _finish("tiny_mixed", 1, 4, 2, 64, 16, q, kv, rng, num_pages=64,
                       max_pages_per_seq=6)
    hq, hkv, d = 32, 8, 128
    if index == 2:
        rng = np.random.default_rng(2)
        n = max(2, int(round(256 * scale)))
        lo, hi = max(2, int(512 * scale)), max(4, int(4096 * scale))
        kv = rng.integers(lo, hi + 1, size=n)
        q = np.ones(n, dtype=np.int64)
        return _finish("decode_256xU512_4096", 2, hq, hkv, d, 16, q, kv, rng)
    if index == 3:
        rng = np.random.default_rng(3)
        n = max(1, int(round(8 * min(1.0, scale * 4))))
        s = max(16, int(2048 * scale))
        q = np.full(n, s, dtype=np.int64)
        return _finish("prefill_8x2048", 3, hq, hkv, d, 16, q, q.copy(), rng)
    if index == 4:
        rng = np.random.default_rng(4)
        nd = max(2, int(round(128 * scale)))
        lo, hi = max(2, int(256 * scale)), max(4, int(8192 * scale))
        kv_d = rng.integers(lo, hi + 1, size=nd)
        chunk = max(4, int(512 * scale))
        ctxs = [max(1, int(c * scale)) for c in (1024, 2048, 4096, 8192)]
        q = np.concatenate([np.ones(nd, dtype=np.int64), np.full(4, chunk, dtype=np.int64)])
        kv = np.concatenate([kv_d, np.asarray(ctxs, dtype=np.int64) + chunk])
        order = rng.permutation(q.shape[0])
        return _finish("mixed_128dec_4x512chunk", 4, hq, hkv, d, 16, q[order], kv[order], rng)
    if index == 5:
        rng = np.random.default_rng(5)
        n = max(2, int(round(32 * min(1.0, scale * 8))))
        lo, hi = 32768 * scale, 131072 * scale
        kv = np.floor(np.exp(rng.uniform(np.log(lo), np.log(hi), size=n))).astype(np.int64)
        kv = np.maximum(kv, 2)
        q = np.ones(n, dtype=np.int64)
        return _finish("long_decode_32xlogU32k_128k", 5, hq, hkv, d, 64, q, kv, rng)
    raise ValueError("config index must be 1..5")


def regime(name: str, hq: int = 32, hkv: int = 8, d: int = 128, ps: int = 16, scale: float = 1.0) -> Workload:
    """The length recipes of configs 2 ("decode"), 3 ("prefill") and 4 ("mixed") at
    any attention shape: the three regimes a set of launch knobs is tuned for."""
    if name == "decode":
        rng = np.random.default_rng(2)
        n = max(2, int(round(256 * scale)))
        kv = rng.integers(max(2, int(512 * scale)), max(4, int(4096 * scale)) + 1, size=n)
        return _finish("regime_decode", 2, hq, hkv, d, ps, np.ones(n, dtype=np.int64), kv, rng)
    if name == "prefill":
        rng = np.random.default_rng(3)
        q = np.full(max(1, int(round(8 * min(1.0, scale * 4)))), max(16, int(2048 * scale)), dtype=np.int64)
        return _finish("regime_prefill", 3, hq, hkv, d, ps, q, q.copy(), rng)
    if name == "mixed":
        rng = np.random.default_rng(4)
        nd = max(2, int(round(128 * scale)))
        kv_d = rng.integers(max(2, int(256 * scale)), max(4, int(8192 * scale)) + 1, size=nd)
        chunk = max(4, int(512 * scale))
        ctxs = [max(1, int(c * scale)) for c in (1024, 2048, 4096, 8192)]
        q = np.concatenate([np.ones(nd, dtype=np.int64), np.full(4, chunk, dtype=np.int64)])
        kv = np.concatenate([kv_d, np.asarray(ctxs, dtype=np.int64) + chunk])
        order = rng.permutation(q.shape[0])
        return _finish("regime_mixed", 4, hq, hkv, d, ps, q[order], kv[order], rng)
    raise ValueError("regime must be decode, prefill or mixed")


def ragged(seed: int, num_seqs: int = 5, hq: int = 4, hkv: int = 2, d: int = 64, ps: int = 16,
           max_q: int = 40, max_ctx: int = 100, spare_pages: int = 3,
           p_decode: float = 0.4, p_empty: float = 0.1) -> Workload:
    """A random small mixed batch: decode rows, prefill rows (ctx 0), chunked
    rows, and some empty (q_len 0) sequences."""
    rng = np.random.default_rng(seed)
    q, kv = [], []
    for _ in range(num_seqs):
        u = rng.random()
        if u < p_empty:
            ql = 0
            ctx = int(rng.integers(0, max_ctx + 1))
        elif u < p_empty + p_decode:
            ql = 1
            ctx = int(rng.integers(0, max_ctx + 1))
        else:
            ql = int(rng.integers(1, max_q + 1))
            ctx = 0 if rng.random() < 0.4 else int(rng.integers(0, max_ctx + 1))
        q.append(ql)
        kv.append(ql + ctx)
    need = int(pages_needed(kv, ps).sum())
    return _finish(f"ragged_seed{seed}", seed, hq, hkv, d, ps, q, kv, rng,
                   num_pages=need + spare_pages)


def uniform(n: int, q_len: int, kv_len: int, hq: int = 32, hkv: int = 8, d: int = 128, ps: int = 256,
            seed: int = 11) -> Workload:
    """n sequences of identical lengths: the shape of the paper's own latency
    tables (Sec. 4.1 decode: n = 128, q_len 1; Sec. 4.2 prefill: n = 1, q_len =
    kv_len; head_dim 128 and 256, page size 256)."""
    rng = np.random.default_rng(seed)
    q = np.full(n, q_len, dtype=np.int64)
    kv = np.full(n, kv_len, dtype=np.int64)
    return _finish(f"uniform_{n}x{q_len}q_{kv_len}kv_d{d}", seed, hq, hkv, d, ps, q, kv, rng)


def live_slot_mask(wl: Workload) -> np.ndarray:
    """bool [num_pages, page_size]: slots holding pre-existing cache content
    (positions < ctx of some sequence).  All other slots are dead before the
    call: either this call writes them or nothing may depend on them."""
    live = np.zeros((wl.num_pages, wl.page_size), dtype=bool)
    ps = wl.page_size
    for r in range(wl.num_seqs):
        ctx = int(wl.kv_lens[r] - wl.q_lens[r])
        full, rem = divmod(ctx, ps)
        if full:
            live[wl.page_table[r, :full]] = True
        if rem:
            live[wl.page_table[r, full], :rem] = True
    return live


def materialize(wl: Workload, device="cpu", poison: bool = True, max_tokens: int | None = None, kv_scales=None):
    """Random bf16 ~ N(0,1) tensors (V clipped to +-3) for the workload, as torch
    tensors on `device`.  With `poison`, every cache slot that is not pre-existing
    content, and every padding token row, holds a NaN bit pattern.

    kv_scales = (k_scale, v_scale): the page pools are uint8 tensors of E4M3
    bytes instead (an 8-bit cache whose stored values stand for value * scale):
    N(0,1) / scale cast with torch's float8_e4m3fn, NaN bytes in dead slots."""
    import torch

    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1000003 * wl.seed + 17)
    t = wl.num_tokens
    tmax = t if max_tokens is None else max_tokens
    assert tmax >= t

    def normal(shape):
        out = torch.empty(shape, dtype=torch.bfloat16, device=dev)
        flat = out.view(-1)
        step = 1 << 26
        for s in range(0, flat.numel(), step):
            n = min(step, flat.numel() - s)
            flat[s:s + n] = torch.randn(n, generator=gen, device=dev, dtype=torch.float32)
        return out

    hq, hkv, d, ps = wl.num_q_heads, wl.num_kv_heads, wl.head_dim, wl.page_size
    q = normal((tmax, hq, d))
    k_new = normal((tmax, hkv, d))
    v_new = normal((tmax, hkv, d))
    k_pages = normal((wl.num_pages, ps, hkv, d))
    v_pages = normal((wl.num_pages, ps, hkv, d))
    # An output row is a convex combination of V rows.  Beyond +-4 the spacing of bf16
    # is 1/32, so a correctly rounded output could miss the fp64 value by up to 1/64,
    # more than a max-abs tolerance of 1.5e-2 allows; it happens where a row sees only
    # a few positions.  |V| <= 3 keeps the rounding of any output under 1/128.
    v_new.clamp_(-3.0, 3.0)
    v_pages.clamp_(-3.0, 3.0)
    if kv_scales is not None:
        def to_bytes(pool, scale):
            x = (pool.float() / float(scale)).clamp_(-448.0, 448.0)
            return x.to(torch.float8_e4m3fn).view(torch.uint8)
        k_pages = to_bytes(k_pages, kv_scales[0])
        v_pages = to_bytes(v_pages, kv_scales[1])
    if poison:
        bad = torch.tensor([POISON_BITS], dtype=torch.int16, device=dev).view(torch.bfloat16)
        dead = torch.from_numpy(~live_slot_mask(wl)).to(dev)
        if kv_scales is not None:
            k_pages[dead] = 0x7F          # the E4M3 NaN byte
            v_pages[dead] = 0x7F
        else:
            k_pages[dead] = bad
            v_pages[dead] = bad
        if tmax > t:
            q[t:] = bad
            k_new[t:] = bad
            v_new[t:] = bad
    return {"q": q, "k_new": k_new, "v_new": v_new, "k_pages": k_pages, "v_pages": v_pages}


def merge_pools(tensors):
    """The same data with the two bf16 page pools laid into one,
    [num_pages, page_size, Hkv, 2, D] (index 0 = K, 1 = V): "kv_pages" replaces
    "k_pages" and "v_pages".  Works on torch tensors and on numpy bit patterns."""
    out = {k: v for k, v in tensors.items() if k not in ("k_pages", "v_pages")}
    k, v = tensors["k_pages"], tensors["v_pages"]
    if isinstance(k, np.ndarray):
        out["kv_pages"] = np.ascontiguousarray(np.stack([k, v], axis=3))
    else:
        import torch

        out["kv_pages"] = torch.stack([k, v], dim=3).contiguous()
    return out


def bits(t):
    """torch bf16 tensor -> numpy uint16 bit patterns (host copy); uint8
    tensors (8-bit cache pools) come back as they are."""
    import torch

    if t.dtype == torch.uint8:
        return t.detach().to("cpu").contiguous().numpy()
    return t.detach().to("cpu").contiguous().view(torch.int16).numpy().view(np.uint16)


# ---------------------------------------------------------------------------
# Discriminating inputs.  With N(0,1) data a long softmax averages thousands of
# rows and an output moves by O(1/kv_len) when one K/V row is wrong, far below
# any tolerance.  The "needle" recipe makes every output row depend on ONE chosen
# position: keys are random sign vectors (entries +-1, so two different keys are
# nearly orthogonal), and the query of (token, head) is twice the key of its
# target position.  The target's score is then sm_scale * 2 * head_dim (22.6 at
# head_dim 128) against N(0, 4 * sm_scale^2 * head_dim) ~ N(0, 2^2) elsewhere, its
# softmax weight is 1 to within 1e-5, and the output row is the target's V row
# (N(0,1) clipped to +-3, distinct per position): a row gathered from a wrong slot, a dropped or
# repeated position or a mask that hides the target changes that output by O(1).
# Only data is built here; which position a query "should" find is decided by
# the softmax of whoever consumes the data.
# ---------------------------------------------------------------------------
def slot_of_position(wl: Workload, r: int, pos):
    """Flat slot index (page * page_size + offset) of positions of sequence r."""
    pos = np.asarray(pos, dtype=np.int64)
    return wl.page_table[r].astype(np.int64)[pos // wl.page_size] * wl.page_size + pos % wl.page_size


def interesting_positions(wl: Workload, r: int, cuts=()):
    """Positions of sequence r where indexing mistakes live: both ends, both sides
    of the first and last page boundary and of every 16- and 64-position tile
    boundary next to them, both sides of the cached/new boundary, both sides of
    every cut in `cuts` (the KV range boundaries a work plan reports)."""
    kv, ql, ps = int(wl.kv_lens[r]), int(wl.q_lens[r]), wl.page_size
    ctx = kv - ql
    cand = {0, 1, 15, 16, 17, 63, 64, 65, ps - 1, ps, ps + 1, kv - 1, kv - 2, ctx - 1, ctx, ctx + 1}
    last_page = ((kv - 1) // ps) * ps
    cand |= {last_page - 1, last_page, last_page + 1, (kv - 1) // 16 * 16 - 1, (kv - 1) // 16 * 16,
             (kv - 1) // 64 * 64 - 1, (kv - 1) // 64 * 64, (ctx // 64) * 64 - 1, (ctx // 64) * 64,
             (ctx // 16) * 16 - 1, (ctx // 16) * 16}
    for c in cuts:
        cand |= {int(c) - 1, int(c)}
    return np.array(sorted(p for p in cand if 0 <= p < kv), dtype=np.int64)


def needle_targets(wl: Workload, mode: str = "spread", seed: int = 0, cuts=None, causal: bool = True) -> np.ndarray:
    """int64 [T, Hq]: the position each (query token, head) is aimed at, always one
    it may see.  mode "spread": the queries of a sequence together visit as many different positions
    of every KV head as they can (all of them once there are kv_len / h_g tokens);
    "boundaries": cycled through interesting_positions(); "random": uniform."""
    rng = np.random.default_rng(7919 * seed + wl.seed)
    hq = wl.num_q_heads
    out = np.zeros((wl.num_tokens, hq), dtype=np.int64)
    cu = wl.cu_q_lens
    for r in range(wl.num_seqs):
        ql, kv = int(wl.q_lens[r]), int(wl.kv_lens[r])
        if ql == 0:
            continue
        ctx = kv - ql
        tok = np.repeat(np.arange(ql, dtype=np.int64), hq)
        visible = (ctx + tok + 1) if causal else np.full(ql * hq, kv, dtype=np.int64)
        k = np.arange(ql * hq, dtype=np.int64)
        if mode == "random":
            t = (rng.random(ql * hq) * visible).astype(np.int64)
        elif mode == "spread":
            # Per KV head: the probes (token, head of the group), taken from the last
            # token backwards, walk down the positions one by one from the last, so
            # that as many different positions as there are probes get visited (each
            # stays visible: the position falls by one per probe, the limit by one per
            # h_g probes); probes left over when position 0 is reached go anywhere.
            hg = hq // wl.num_kv_heads
            j = (k % hq) % hg                                    # head inside its group
            kk = (ql - 1 - tok) * hg + (j + seed) % hg           # probe index inside the KV head
            t = np.where(kk < kv, kv - 1 - kk, (rng.random(ql * hq) * visible).astype(np.int64))
            t = np.minimum(t, visible - 1)
        elif mode == "boundaries":
            pts = interesting_positions(wl, r, cuts[r] if cuts is not None else ())
            shift = int(rng.integers(0, len(pts)))
            t = pts[(k + shift) % len(pts)]
            hidden = t >= visible                       # aimed past the token's own position: take its last one
            t = np.where(hidden, visible - 1 - (k % np.minimum(visible, 3)), t)
        else:
            raise ValueError("mode must be spread, boundaries or random")
        out[cu[r]:cu[r + 1]] = np.minimum(t, visible - 1).reshape(ql, hq)
    return out


def materialize_needles(wl: Workload, targets: np.ndarray, device="cpu", poison: bool = True,
                        max_tokens: int | None = None, kv_scales=None):
    """Like materialize(), with sign-vector keys and queries aimed at `targets`
    (needle_targets()).  V, and everything about poison and padding, as there."""
    import torch

    dev = torch.device(device)
    x = materialize(wl, dev, poison=False, max_tokens=max_tokens, kv_scales=None)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1000003 * wl.seed + 29)

    def signs(like):
        flat = like.view(-1)
        step = 1 << 26
        for s in range(0, flat.numel(), step):
            n = min(step, flat.numel() - s)
            flat[s:s + n] = (torch.randint(0, 2, (n,), generator=gen, device=dev, dtype=torch.int8) * 2 - 1).to(like.dtype)
        return like

    signs(x["k_pages"])
    signs(x["k_new"])
    # (V is clipped to +-3 by materialize(): an output row here is one V row)
    hq, hkv, d, ps = wl.num_q_heads, wl.num_kv_heads, wl.head_dim, wl.page_size
    hg = hq // hkv
    t_total = wl.num_tokens
    if t_total:
        # source row of every (token, head): a slot of the page pool or a row of k_new
        cu = wl.cu_q_lens
        is_new = np.zeros((t_total, hq), dtype=bool)
        row = np.zeros((t_total, hq), dtype=np.int64)
        for r in range(wl.num_seqs):
            ql = int(wl.q_lens[r])
            if ql == 0:
                continue
            ctx = int(wl.kv_lens[r]) - ql
            t = targets[cu[r]:cu[r + 1]]
            new = t >= ctx
            is_new[cu[r]:cu[r + 1]] = new
            row[cu[r]:cu[r + 1]] = np.where(new, cu[r] + t - ctx, slot_of_position(wl, r, np.where(new, 0, t)))
        g_of_h = torch.arange(hq, device=dev) // hg
        row_t = torch.from_numpy(row).to(dev)
        new_t = torch.from_numpy(is_new).to(dev)
        pool = x["k_pages"].view(wl.num_pages * ps, hkv, d)
        from_pool = pool[row_t.clamp(max=wl.num_pages * ps - 1), g_of_h[None, :]]        # [T, Hq, D]
        from_new = x["k_new"][row_t.clamp(max=x["k_new"].shape[0] - 1), g_of_h[None, :]]
        x["q"][:t_total] = 2.0 * torch.where(new_t[..., None], from_new, from_pool)
    if kv_scales is not None:
        def to_bytes(pool, scale):
            v = (pool.float() / float(scale)).clamp_(-448.0, 448.0)
            return v.to(torch.float8_e4m3fn).view(torch.uint8)
        x["k_pages"] = to_bytes(x["k_pages"], kv_scales[0])
        x["v_pages"] = to_bytes(x["v_pages"], kv_scales[1])
    if poison:
        bad = torch.tensor([POISON_BITS], dtype=torch.int16, device=dev).view(torch.bfloat16)
        dead = torch.from_numpy(~live_slot_mask(wl)).to(dev)
        if kv_scales is not None:
            x["k_pages"][dead] = 0x7F
            x["v_pages"][dead] = 0x7F
        else:
            x["k_pages"][dead] = bad
            x["v_pages"][dead] = bad
        tmax = x["q"].shape[0]
        if tmax > t_total:
            for name in ("q", "k_new", "v_new"):
                x[name][t_total:] = bad
    return x
