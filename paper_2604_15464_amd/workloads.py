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
    """Random bf16 ~ N(0,1) tensors for the workload, as torch tensors on
    `device`.  With `poison`, every cache slot that is not pre-existing
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


def bits(t):
    """torch bf16 tensor -> numpy uint16 bit patterns (host copy); uint8
    tensors (8-bit cache pools) come back as they are."""
    import torch

    if t.dtype == torch.uint8:
        return t.detach().to("cpu").contiguous().numpy()
    return t.detach().to("cpu").contiguous().view(torch.int16).numpy().view(np.uint16)
