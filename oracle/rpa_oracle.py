"""CPU oracle for ragged paged attention with fused KV-cache update.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
HIP path is checked against.  It shares no code with the HIP path, is never
imported by the product package, and must never be used as a fallback.

What it computes (paper Sec. 3, Algorithm 1 "RPA Forward Pass with KV Cache
Update Fusion"): for every sequence r of a ragged batch, the newly projected
K/V rows are written into the paged cache at the sequence's last l_q
positions (Alg. 1, the "update new KV entries" step; Sec. 3.3 "Update U_kv"),
and every query token attends causally over the sequence's cached plus new KV
(Alg. 1 inner loop).  The FlashAttention-2 recurrences of Alg. 1 (running max
m, running sum l, rescaled accumulator, final diag(l)^-1) reach exactly plain
softmax attention, and paging only changes addressing, so the oracle is the
plain definition written out: scatter, explicit gather to contiguous arrays,
dense masked two-pass softmax in fp64.  No tiling, no online softmax.

Readings where the paper is silent (each also listed in the design notes):
  * scores are sm_scale * (q . k); sm_scale is the fp32 value of the call,
    promoted to fp64 (Alg. 1 writes S = C_q C_k^T without a scale);
  * "mask S if needed" (Alg. 1) is the causal mask aligned to the end of the
    sequence: query i (0-based in its sequence) sees positions
    j <= kv_len - q_len + i; with causal=False (the paper's non-causal prefill
    measurements, Sec. 4.2) every query sees all kv_len positions, its own
    sequence's later tokens included;
  * kv_len counts this call's new tokens (Sec. 4.1 defines the context
    length as covering cached and newly projected KV alike);
  * query head h reads KV head h // (Hq / Hkv) (Sec. 3.1.2: the h_g heads of
    a group are stacked against one K/V operand);
  * the result is as if the update finished before attention starts.

Pins (tests/test_oracle_pins.py, all CPU): pure-Python brute force on
contiguous KV, page-permutation invariance, decode == last prefill row,
chunk composition across calls, torch's float64 scaled_dot_product_attention
on the contiguous single-sequence case, closed forms (constant V, equal K,
hand-built log-weights, shift invariance), the split-merge identity, sentinel
bytes, idempotence; for the 8-bit cache torch's float8_e4m3fn casts, a
nearest-neighbour search over the 256 decoded values, the lossless case and
power-of-two scale invariance; for the merged pool the pure-Python brute force
on a pool filled token by token, and equality with the two-pool call.  No
function here is "parity unpinned".
"""
from __future__ import annotations

import math

import numpy as np


# --------------------------------------------------------------------------
# bf16 <-> fp64 (exact decode; round-to-nearest-even encode)
# --------------------------------------------------------------------------
def bf16_to_f64(u16: np.ndarray) -> np.ndarray:
    """Exact value of bf16 bit patterns: the pattern is the top half of an
    IEEE float32."""
    u32 = np.asarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    with np.errstate(invalid="ignore"):       # signalling-NaN patterns are legal input
        return u32.view(np.float32).astype(np.float64)


def f64_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp64 -> fp32 -> bf16 (nearest even), returned as bit patterns.
    Only used to report a rounded copy of the oracle output."""
    f32 = np.asarray(x, dtype=np.float64).astype(np.float32)
    u32 = f32.view(np.uint32)
    lsb = (u32 >> np.uint32(16)) & np.uint32(1)
    rounded = (u32 + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    out = rounded.astype(np.uint16)
    nan = np.isnan(f32)
    out[nan] = 0x7FC0
    return out


# --------------------------------------------------------------------------
# 8-bit KV cache (Sec. 3.6 "Quantization": per-tensor scaling, one scalar per
# tensor).  The paper names FP8 but neither the encoding nor the rounding; the
# reading taken here: OCP E4M3 ("fn": sign, 4 exponent bits with bias 7, 3
# mantissa bits, subnormals, no infinities, 0x7f / 0xff = NaN, largest finite
# value 448), a stored byte b stands for value(b) * scale, and a new row x is
# stored as the byte nearest (ties to even) to fp32(x) * fp32(1 / scale),
# saturated to +-448, both operations in fp32.
# --------------------------------------------------------------------------
E4M3_MAX = 448.0


def e4m3_to_f64(u8: np.ndarray) -> np.ndarray:
    """Exact value of E4M3 bytes."""
    b = np.asarray(u8, dtype=np.uint8).astype(np.int64)
    sign = np.where(b & 0x80, -1.0, 1.0)
    e = (b >> 3) & 0xF
    m = (b & 0x7).astype(np.float64)
    val = np.where(e == 0, m / 8.0 * 2.0 ** -6, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))
    val = sign * val
    return np.where((b & 0x7F) == 0x7F, np.nan, val)


def f32_to_e4m3(x: np.ndarray) -> np.ndarray:
    """fp32 -> nearest E4M3 byte, ties to the even mantissa, saturating at
    +-448.  (NaN gives a NaN byte; which of the two is not specified.)"""
    x = np.asarray(x, dtype=np.float32)
    a = np.minimum(np.abs(x.astype(np.float64)), E4M3_MAX)
    sign = np.signbit(x).astype(np.int64) << 7
    frac, expo = np.frexp(a)                       # a = frac * 2**expo, frac in [0.5, 1)
    e_unb = np.maximum(expo - 1, -6)               # below 2**-6 the grid of the subnormals continues
    step = np.exp2((e_unb - 3).astype(np.float64))  # spacing of representable values in this binade
    with np.errstate(invalid="ignore"):            # NaN input (padding rows) is handled below
        q = np.rint(a / step).astype(np.int64)     # numpy rounds halves to even; q in [0, 16]
    carry = q == 16                                # rounded up into the next binade
    e_unb = np.where(carry, e_unb + 1, e_unb)
    q = np.where(carry, 8, q)
    normal = q >= 8
    code = np.where(normal, ((e_unb + 7) << 3) | (q - 8), q)   # subnormal: exponent field 0, mantissa q
    code = np.where(np.isnan(x), 0x7F, code)
    return (sign | code).astype(np.uint8)


def quantize_rows(new_u16: np.ndarray, scale: float) -> np.ndarray:
    """bf16 bit patterns -> E4M3 bytes of value / scale."""
    inv = np.float32(1.0) / np.float32(scale)
    x32 = (np.asarray(new_u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
    return f32_to_e4m3(x32 * inv)                  # fp32 product, rounded to nearest


# --------------------------------------------------------------------------
# step 1: cache update (bit copy)
# --------------------------------------------------------------------------
def update_cache(k_new, v_new, k_pages, v_pages, page_table, cu_q_lens, kv_lens, num_seqs):
    """Write the new rows of every sequence into its pages, in place.

    k_new, v_new : uint16 [T, Hkv, D];  k_pages, v_pages : uint16 [P, ps, Hkv, D]
    Token t of sequence r (0 <= t < l_q) lands at position ctx + t, i.e. in
    page page_table[r][pos // ps], slot pos % ps.
    """
    ps = k_pages.shape[1]
    for r in range(num_seqs):
        q0 = int(cu_q_lens[r])
        l_q = int(cu_q_lens[r + 1]) - q0
        l_kv = int(kv_lens[r])
        ctx = l_kv - l_q
        if l_q < 0 or ctx < 0:
            raise ValueError("bad lengths")
        for t in range(l_q):
            pos = ctx + t
            pg = int(page_table[r, pos // ps])
            if pg < 0:
                raise ValueError("page table entry missing")
            k_pages[pg, pos % ps] = k_new[q0 + t]
            v_pages[pg, pos % ps] = v_new[q0 + t]


# --------------------------------------------------------------------------
# step 2: explicit gather of one sequence's KV
# --------------------------------------------------------------------------
def gather_sequence(pages, table_row, l_kv):
    """pages uint16 [P, ps, Hkv, D] -> contiguous uint16 [l_kv, Hkv, D]."""
    ps = pages.shape[1]
    n_pages = (l_kv + ps - 1) // ps
    ids = np.asarray(table_row[:n_pages], dtype=np.int64)
    if (ids < 0).any():
        raise ValueError("page table entry missing")
    flat = pages[ids].reshape(n_pages * ps, pages.shape[2], pages.shape[3])
    return flat[:l_kv]


# --------------------------------------------------------------------------
# step 3: dense causal GQA softmax attention of one sequence, fp64, two-pass
# --------------------------------------------------------------------------
def attend_sequence(q, k, v, sm_scale, heads=None, causal=True):
    """q fp64 [l_q, Hq, D]; k, v fp64 [l_kv, Hkv, D] -> fp64 [l_q, Hq, D].

    The last l_q positions of k/v are the queries' own tokens."""
    l_q, hq, d = q.shape
    l_kv, hkv, _ = k.shape
    hg = hq // hkv
    ctx = l_kv - l_q
    scale = float(np.float32(sm_scale))
    out = np.zeros((l_q, hq, d), dtype=np.float64)
    i = np.arange(l_q)[:, None]
    j = np.arange(l_kv)[None, :]
    hidden = (j > (ctx + i)) if causal else np.zeros((l_q, l_kv), dtype=bool)
    for h in (range(hq) if heads is None else heads):
        g = h // hg
        s = scale * (q[:, h, :] @ k[:, g, :].T)
        s[hidden] = -np.inf
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ v[:, g, :]
    return out


# --------------------------------------------------------------------------
# the whole call
# --------------------------------------------------------------------------
def update_and_attend(q, k_new, v_new, k_pages, v_pages, page_table, cu_q_lens, kv_lens,
                      num_seqs, sm_scale, seqs=None, heads=None, causal=True, kv_scales=None):
    """The oracle of the library call.

    All tensor arguments are numpy uint16 arrays of bf16 bit patterns.
    Returns (out fp64 [T, Hq, D], k_pages', v_pages').  The input pools are
    not modified.  `seqs` restricts the attention part (not the update) to
    some sequences, for sampled checks at large sizes; rows of other
    sequences are NaN.

    kv_scales = (k_scale, v_scale) selects the 8-bit cache: the pools are
    uint8 arrays of E4M3 bytes, the new rows are quantised on their way in
    and attention reads value(byte) * scale for every position, this call's
    own tokens included (the result is as if the update finished first).
    """
    if kv_scales is not None:
        k_scale, v_scale = (float(np.float32(s)) for s in kv_scales)
        k_pages = np.array(k_pages, dtype=np.uint8, copy=True)
        v_pages = np.array(v_pages, dtype=np.uint8, copy=True)
        update_cache(quantize_rows(k_new, k_scale), quantize_rows(v_new, v_scale), k_pages, v_pages, page_table,
                     cu_q_lens, kv_lens, num_seqs)
        decode_k = lambda u: e4m3_to_f64(u) * k_scale
        decode_v = lambda u: e4m3_to_f64(u) * v_scale
    else:
        k_pages = np.array(k_pages, dtype=np.uint16, copy=True)
        v_pages = np.array(v_pages, dtype=np.uint16, copy=True)
        update_cache(k_new, v_new, k_pages, v_pages, page_table, cu_q_lens, kv_lens, num_seqs)
        decode_k = decode_v = bf16_to_f64
    t_total = int(cu_q_lens[num_seqs]) if num_seqs > 0 else 0
    out = np.full((q.shape[0], q.shape[1], q.shape[2]), np.nan, dtype=np.float64)
    for r in (range(num_seqs) if seqs is None else seqs):
        q0 = int(cu_q_lens[r])
        l_q = int(cu_q_lens[r + 1]) - q0
        if l_q == 0:
            continue
        l_kv = int(kv_lens[r])
        kk = decode_k(gather_sequence(k_pages, page_table[r], l_kv))
        vv = decode_v(gather_sequence(v_pages, page_table[r], l_kv))
        qq = bf16_to_f64(q[q0:q0 + l_q])
        res = attend_sequence(qq, kk, vv, sm_scale, heads=heads, causal=causal)
        if heads is None:
            out[q0:q0 + l_q] = res
        else:
            hs = list(heads)
            out[q0:q0 + l_q, hs] = res[:, hs]
    assert t_total <= q.shape[0]
    return out, k_pages, v_pages


# --------------------------------------------------------------------------
# the merged KV layout (Sec. 3.1.3 "KV merge"): one pool in which the K and the
# V row of a token and head lie side by side.  Only addressing changes.  The
# paper interleaves at the granularity its hardware packs rows in; the reading
# here keeps whole rows: pool uint16 [P, ps, Hkv, 2, D], index 0 = K, 1 = V.
# --------------------------------------------------------------------------
def update_and_attend_merged(q, k_new, v_new, kv_pages, page_table, cu_q_lens, kv_lens, num_seqs, sm_scale,
                             seqs=None, heads=None, causal=True):
    """As update_and_attend on a merged pool.  Returns (out, kv_pages')."""
    kv_pages = np.array(kv_pages, dtype=np.uint16, copy=True)
    ps = kv_pages.shape[1]
    for r in range(num_seqs):
        q0 = int(cu_q_lens[r])
        l_q = int(cu_q_lens[r + 1]) - q0
        ctx = int(kv_lens[r]) - l_q
        if l_q < 0 or ctx < 0:
            raise ValueError("bad lengths")
        for t in range(l_q):
            pg = int(page_table[r, (ctx + t) // ps])
            if pg < 0:
                raise ValueError("page table entry missing")
            kv_pages[pg, (ctx + t) % ps, :, 0, :] = k_new[q0 + t]
            kv_pages[pg, (ctx + t) % ps, :, 1, :] = v_new[q0 + t]
    out = np.full(q.shape, np.nan, dtype=np.float64)
    for r in (range(num_seqs) if seqs is None else seqs):
        q0 = int(cu_q_lens[r])
        l_q = int(cu_q_lens[r + 1]) - q0
        if l_q == 0:
            continue
        l_kv = int(kv_lens[r])
        n_pages = (l_kv + ps - 1) // ps
        rows = kv_pages[np.asarray(page_table[r, :n_pages], dtype=np.int64)]      # [n_pages, ps, Hkv, 2, D]
        rows = rows.reshape(n_pages * ps, *kv_pages.shape[2:])[:l_kv]
        res = attend_sequence(bf16_to_f64(q[q0:q0 + l_q]), bf16_to_f64(rows[:, :, 0, :]), bf16_to_f64(rows[:, :, 1, :]),
                              sm_scale, heads=heads, causal=causal)
        if heads is None:
            out[q0:q0 + l_q] = res
        else:
            hs = list(heads)
            out[q0:q0 + l_q, hs] = res[:, hs]
    return out, kv_pages


# --------------------------------------------------------------------------
# merge rule for partial results over disjoint KV ranges
# --------------------------------------------------------------------------
def partial_attention(q_row, k, v, scale):
    """Un-normalised partial of one query row over a KV range:
    (m, l, o) with m = max score, l = sum exp(s - m), o = sum exp(s - m) v.
    An empty range gives (-inf, 0, 0)."""
    if k.shape[0] == 0:
        return -np.inf, 0.0, np.zeros(v.shape[1], dtype=np.float64)
    s = scale * (k @ q_row)
    m = float(s.max())
    p = np.exp(s - m)
    return m, float(p.sum()), p @ v


def merge_partials(parts):
    """Combine (m, l, o) partials of disjoint ranges (follows from the
    rescaling step of Alg. 1: states with different running maxima are
    brought to the common maximum before they are added)."""
    big = max(m for m, _, _ in parts)
    num = 0.0
    den = 0.0
    for m, l, o in parts:
        w = 0.0 if m == -np.inf else math.exp(m - big)
        num = num + w * o
        den = den + w * l
    return num / den


# --------------------------------------------------------------------------
# structurally different brute force, for pinning the above on tiny inputs
# --------------------------------------------------------------------------
def dense_bruteforce(q, k, v, sm_scale, causal=True):
    """Pure-Python triple loop over contiguous lists.

    q: [l_q][Hq][D], k/v: [l_kv][Hkv][D] nested lists (or arrays) of floats;
    the queries are the last l_q positions.  Returns nested lists."""
    l_q, hq, d = len(q), len(q[0]), len(q[0][0])
    l_kv, hkv = len(k), len(k[0])
    hg = hq // hkv
    ctx = l_kv - l_q
    scale = float(np.float32(sm_scale))
    out = [[[0.0] * d for _ in range(hq)] for _ in range(l_q)]
    for i in range(l_q):
        last = ctx + i if causal else l_kv - 1
        for h in range(hq):
            g = h // hg
            scores = []
            for j in range(last + 1):
                acc = 0.0
                for c in range(d):
                    acc += float(q[i][h][c]) * float(k[j][g][c])
                scores.append(scale * acc)
            top = max(scores)
            w = [math.exp(s - top) for s in scores]
            z = math.fsum(w)
            for c in range(d):
                out[i][h][c] = math.fsum(w[j] * float(v[j][g][c]) for j in range(last + 1)) / z
    return out
