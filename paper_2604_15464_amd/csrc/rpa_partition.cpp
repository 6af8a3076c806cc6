// Host-side work partitioner and kernel-variant selector.
//
// Algorithm 1 of the paper walks sequences, Q blocks and KV blocks serially on
// one core.  Here the same iteration space is flattened into independent units
// (sequence, Q tile, KV range) so that 256 compute units stay busy: a tile whose
// KV range is long is cut into several ranges whose partial softmax states are
// merged afterwards.  Narrow (bandwidth-bound) units are dealt into bins of
// equal KV volume, one resident workgroup per bin, by cutting the concatenated
// KV stream of all narrow tiles at equal intervals; wide (MFMA-bound) units are
// one workgroup each, longest first.  The regime split of Sec. 3.4
// (decode-only / prefill-only / mixed) becomes a per-sequence choice between
// the narrow and the wide kernel.
#include <algorithm>
#include <cstdio>

#include <cmath>

#include "rpa_internal.h"

namespace rpa {

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

int check_shape(const rpa_shape& s, std::string& err) {
    char buf[256];
    if (s.num_q_heads <= 0 || s.num_kv_heads <= 0 || s.head_dim <= 0 || s.page_size <= 0 ||
        s.max_tokens <= 0 || s.max_seqs <= 0 || s.max_pages_per_seq <= 0 || s.num_pages <= 0) {
        err = "shape fields must all be positive";
        return RPA_ERR_INVALID_ARG;
    }
    if (s.head_dim != 64 && s.head_dim != 128 && s.head_dim != 256) {
        snprintf(buf, sizeof buf, "head_dim %d unsupported (64, 128 or 256)", s.head_dim);
        err = buf;
        return RPA_ERR_UNSUPPORTED;
    }
    if (s.num_q_heads % s.num_kv_heads != 0 || narrow_q_tokens(s.num_q_heads / s.num_kv_heads) == 0) {
        snprintf(buf, sizeof buf, "num_q_heads %d / num_kv_heads %d: group size must be 1, 2, 4, 8 or 16",
                 s.num_q_heads, s.num_kv_heads);
        err = buf;
        return RPA_ERR_UNSUPPORTED;
    }
    if (s.page_size < 16 || (s.page_size & (s.page_size - 1)) != 0) {
        snprintf(buf, sizeof buf, "page_size %d unsupported (power of two, at least 16)", s.page_size);
        err = buf;
        return RPA_ERR_UNSUPPORTED;
    }
    if (s.kv_fp8 != 0 && s.kv_fp8 != 1) {
        err = "kv_fp8 must be 0 or 1";
        return RPA_ERR_INVALID_ARG;
    }
    if (s.kv_fp8 && !(s.k_scale > 0.f && s.v_scale > 0.f && std::isfinite(s.k_scale) && std::isfinite(s.v_scale) &&
                      std::isfinite(1.f / s.k_scale) && std::isfinite(1.f / s.v_scale))) {
        err = "k_scale and v_scale must be positive and finite, and so must their reciprocals";
        return RPA_ERR_INVALID_ARG;
    }
    if (s.kv_merged != 0 && s.kv_merged != 1) {
        err = "kv_merged must be 0 or 1";
        return RPA_ERR_INVALID_ARG;
    }
    if (s.kv_merged && (s.kv_fp8 || s.head_dim != 128)) {
        err = "the merged K|V pool is built for a bf16 cache at head_dim 128";
        return RPA_ERR_UNSUPPORTED;
    }
    if ((int64_t)s.num_pages * s.page_size * s.num_kv_heads * s.head_dim >= ((int64_t)1 << 40)) {
        err = "page pool too large";
        return RPA_ERR_UNSUPPORTED;
    }
    return RPA_OK;
}

int classify_batch(const rpa_shape& s, const int32_t* cu, int32_t n) {
    const int hg = s.num_q_heads / s.num_kv_heads;
    const int64_t narrow_max_q = narrow_q_tokens(hg); // one narrow tile, as in build_plan
    const bool narrow_only = (s.kv_fp8 && s.head_dim != 128) || s.kv_merged;
    bool any_narrow = false, any_wide = false;
    for (int32_t r = 0; r < n; ++r) {
        const int64_t lq = (int64_t)cu[r + 1] - cu[r];
        if (lq <= 0) continue;
        ((!narrow_only && lq > narrow_max_q) ? any_wide : any_narrow) = true;
    }
    return any_wide ? (any_narrow ? RPA_VARIANT_MIXED : RPA_VARIANT_PREFILL) : RPA_VARIANT_DECODE;
}

namespace {

struct Tile {
    int32_t seq, q_pos0, n_q, kv_hi, ctx, seq_q0;
    bool wide;
    bool alone; // the only query tile of its sequence: no other tile reads these K/V rows
};

void emit_units(const Tile& t, int64_t chunk, int align, int num_q_heads, int64_t& part_cursor,
                std::vector<rpa_work_unit>& units, std::vector<rpa_combine_item>& items,
                int32_t& max_splits) {
    int64_t n_s = std::max<int64_t>(1, ceil_div(t.kv_hi, chunk));
    int64_t per = round_up(ceil_div(t.kv_hi, n_s), align);
    n_s = ceil_div(t.kv_hi, per);
    const int32_t rows = t.n_q * num_q_heads;
    int32_t base = -1;
    if (n_s > 1) {
        base = (int32_t)part_cursor;
        part_cursor += n_s * rows;
        items.push_back(rpa_combine_item{base, (int32_t)n_s, rows, t.seq_q0 + t.q_pos0});
    }
    max_splits = std::max<int32_t>(max_splits, (int32_t)n_s);
    for (int64_t s = 0; s < n_s; ++s) {
        rpa_work_unit u{};
        u.seq = t.seq;
        u.q_start = t.seq_q0 + t.q_pos0;
        u.q_pos0 = t.q_pos0;
        u.n_q = t.n_q;
        u.kv_begin = (int32_t)(s * per);
        u.kv_end = (int32_t)std::min<int64_t>((s + 1) * per, t.kv_hi);
        u.ctx = t.ctx;
        u.seq_q0 = t.seq_q0;
        u.part_row = n_s > 1 ? (int32_t)(base + s * rows) : -1;
        u.flags = (s == n_s - 1 ? 1 : 0) | (t.wide ? 2 : 0) | (t.alone ? 4 : 0);
        units.push_back(u);
    }
}

} // namespace

int build_plan(const rpa_shape& s, const int32_t* cu, const int32_t* kv, int32_t n,
               const rpa_options& opt, int num_cus, int64_t partial_row_cap, Plan& plan,
               std::string& err) {
    char buf[256];
    plan.narrow.clear();
    plan.wide.clear();
    plan.items.clear();
    plan.stats = rpa_plan_stats{};
    if (n < 0 || n > s.max_seqs) {
        snprintf(buf, sizeof buf, "num_seqs %d outside [0, max_seqs=%d]", n, s.max_seqs);
        err = buf;
        return RPA_ERR_BAD_LENGTHS;
    }
    if (opt.variant < RPA_VARIANT_AUTO || opt.variant > RPA_VARIANT_MIXED || opt.kv_chunk < 0 ||
        opt.wide_kv_chunk < 0 || opt.units_per_cu < 0 || opt.narrow_waves < 0 || opt.narrow_waves > kMaxWaves ||
        (opt.narrow_waves > 0 && s.num_kv_heads % opt.narrow_waves != 0) ||
        (opt.wide_rows != 0 && opt.wide_rows != 128 && opt.wide_rows != 256) || opt.wide_order < 0 ||
        opt.wide_order > 2 || opt.mixed_overlap < 0 || opt.mixed_overlap > 3 || opt.stream_ordered_upload < 0 ||
        opt.stream_ordered_upload > 3 || opt.wide_persistent < 0 || opt.wide_persistent > 1 ||
        !options_fit_shape(s, opt)) {
        err = "bad options";
        return RPA_ERR_INVALID_ARG;
    }
    if (n > 0 && (!cu || !kv)) {
        err = "cu_q_lens / kv_lens is null";
        return RPA_ERR_INVALID_ARG;
    }
    if (n > 0 && cu[0] != 0) {
        err = "cu_q_lens[0] must be 0";
        return RPA_ERR_BAD_LENGTHS;
    }
    const int hg = s.num_q_heads / s.num_kv_heads;
    const int tq_narrow = narrow_q_tokens(hg);
    for (int32_t r = 0; r < n; ++r) {
        const int64_t lq = (int64_t)cu[r + 1] - cu[r];
        if (lq < 0) {
            snprintf(buf, sizeof buf, "cu_q_lens decreases at sequence %d", r);
            err = buf;
            return RPA_ERR_BAD_LENGTHS;
        }
        if (cu[r + 1] > s.max_tokens) {
            snprintf(buf, sizeof buf, "more than max_tokens=%d packed tokens", s.max_tokens);
            err = buf;
            return RPA_ERR_BAD_LENGTHS;
        }
        if (kv[r] < lq) {
            snprintf(buf, sizeof buf, "sequence %d: kv_len %d < q_len %lld", r, kv[r], (long long)lq);
            err = buf;
            return RPA_ERR_BAD_LENGTHS;
        }
        if (ceil_div(kv[r], s.page_size) > s.max_pages_per_seq) {
            snprintf(buf, sizeof buf, "sequence %d: kv_len %d needs more than max_pages_per_seq=%d pages", r,
                     kv[r], s.max_pages_per_seq);
            err = buf;
            return RPA_ERR_BAD_LENGTHS;
        }
    }

    // ---- regime per sequence (Sec. 3.4) ---------------------------------
    // Narrow up to one narrow tile of query tokens (16 / h_g): a second tile would
    // stream the sequence's K/V a second time (256 sequences of 8 tokens on 2 K of
    // context at h_g 4: 683 us narrow, 495 us wide).
    const int64_t narrow_max_q = tq_narrow;
    // the 8-bit cache has a wide kernel at head_dim 128 only; elsewhere, and with the
    // merged K|V pool, every batch runs narrow
    const bool narrow_only = (s.kv_fp8 && s.head_dim != 128) || s.kv_merged;
    // Wide tile height: 256 rows (half the K/V staging traffic per row, no stall
    // on the loads) when that still gives every CU several workgroups, else 128
    // rows (twice as many, independent workgroups).
    int wide_rows = opt.wide_rows;
    if (s.head_dim > 128) {
        wide_rows = kWideRows; // the only shape built for this head_dim
    } else if (wide_rows == 0 && s.head_dim == 64) {
        // head_dim 64: a 4-wave workgroup takes 112 registers per lane and 32 KB of LDS,
        // so four of them share a CU (four waves per SIMD), which hides the softmax
        // behind the MFMAs far better than one 8-wave workgroup (8 x 2048: 160 against
        // 199 us, 16 x 1024: 90 against 118 us; one long sequence: the same)
        wide_rows = kWideRows;
    } else if (wide_rows == 0 && s.kv_fp8) {
        // 8-bit cache: the widening of the operands makes the loop heavier in vector
        // work, and two independent 4-wave workgroups per CU hide that better than one
        // of eight waves (8 x 2048: 333 against 361 us, one 16 K sequence: 2274
        // against 2376 us; one 4 K sequence: 175 against 172 us)
        wide_rows = kWideRows;
    } else if (wide_rows == 0) {
        // 256 rows also when there is one workgroup per CU and the items are long and
        // full: such a launch is bound by throughput, where the 8-wave shape moves
        // half the K/V per row (16 chunks of 128 tokens on 8 K of context: 285 against
        // 318 us; 32 of 64 tokens on 4 K: 163 against 178 us), while short items are
        // bound by their own length and run better as twice as many workgroups (8
        // chunks of 256 on 2 K: 80 against 91 us; one 4 K sequence: 144 against 150 us).
        int64_t tiles256 = 0, work256 = 0, tokens = 0;
        bool narrow_beside = false;
        const int32_t tq256 = wide_q_tokens(hg, 256);
        for (int32_t r = 0; r < n; ++r) {
            const int32_t lq = cu[r + 1] - cu[r];
            const bool wide = !narrow_only && (opt.variant == RPA_VARIANT_PREFILL ||
                                               (opt.variant != RPA_VARIANT_DECODE && lq > narrow_max_q));
            if (lq > 0 && !wide) narrow_beside = true;
            if (lq <= 0 || !wide) continue;
            tiles256 += ceil_div(lq, tq256);
            tokens += lq;
            for (int32_t i0 = 0; i0 < lq; i0 += tq256)
                work256 += s.non_causal ? kv[r] : kv[r] - lq + std::min(lq, i0 + tq256);
        }
        const int64_t cus1 = std::max(1, num_cus);
        // (and tiles that the sequences fill to three quarters at least: 512 prefills of
        // 32 tokens half-fill 256-row tiles, 99 against 71 us with 128-row ones)
        const bool many = tiles256 * s.num_kv_heads >= 4 * cus1 && tokens * 4 >= tiles256 * tq256 * 3;
        const bool long_and_full = tiles256 * s.num_kv_heads >= cus1 && work256 >= tiles256 * 64 * kWideKvTile &&
                                   tokens * 10 >= tiles256 * tq256 * 9;
        // beside narrow work: 128 rows, the shape that shares a CU and a launch with
        // narrow workgroups (64 decode sequences + 8 x 2048 prefill: 367 us against 389
        // us as two kernels with 256-row tiles; 128 + one 8 K prefill: 756 / 837 us)
        wide_rows = (!narrow_beside && (many || long_and_full)) ? 256 : kWideRows;
    }
    bool any_narrow = false, any_wide = false;
    std::vector<Tile> tiles;
    int64_t work_wide = 0, wide_tiles = 0, longest_wide = 0; // KV positions of all wide tiles, their number, the longest
    for (int32_t r = 0; r < n; ++r) {
        const int32_t lq = cu[r + 1] - cu[r];
        if (lq == 0) continue;
        bool wide;
        switch (narrow_only ? RPA_VARIANT_DECODE : opt.variant) {
        case RPA_VARIANT_DECODE: wide = false; break;
        case RPA_VARIANT_PREFILL: wide = true; break;
        default: wide = lq > narrow_max_q; break;
        }
        (wide ? any_wide : any_narrow) = true;
        const int32_t ctx = kv[r] - lq;
        const int32_t tq = wide ? wide_q_tokens(hg, wide_rows) : tq_narrow;
        for (int32_t i0 = 0; i0 < lq; i0 += tq) {
            Tile t{r, i0, std::min(tq, lq - i0), 0, ctx, cu[r], wide, lq <= tq};
            t.kv_hi = s.non_causal ? kv[r] : ctx + i0 + t.n_q; // last position any row of the tile sees, + 1
            tiles.push_back(t);
            if (wide) {
                work_wide += t.kv_hi;
                longest_wide = std::max<int64_t>(longest_wide, t.kv_hi);
                ++wide_tiles;
            }
        }
    }
    plan.stats.variant = any_wide ? (any_narrow ? RPA_VARIANT_MIXED : RPA_VARIANT_PREFILL) : RPA_VARIANT_DECODE;

    // ---- narrow units: equal-volume bins -------------------------------------
    // The narrow kernel keeps `slots` workgroups resident (LDS-bound); each gets
    // one bin and walks its pieces back to back, so every workgroup streams the
    // same number of KV tiles and there is no tail.
    const int cus = std::max(1, num_cus);
    int64_t total_tiles = 0; // KV volume of all narrow tiles, in 16-position tiles
    for (const Tile& t : tiles)
        if (!t.wide) total_tiles += ceil_div(t.kv_hi, kNarrowKvTile);

    // Narrow and wide kernels side by side when both parts are worth more than the
    // extra stream packets (about 10 us): the narrow kernel is bound by HBM, the
    // wide one by the matrix and vector pipes, and a CU holds a workgroup of each.
    bool concurrent = false;
    const double kv_elem_bytes = s.kv_fp8 ? 1.0 : 2.0;
    const double narrow_bytes = (double)total_tiles * kNarrowKvTile * s.num_kv_heads * s.head_dim * 2.0 * kv_elem_bytes;
    const double wide_flops = (double)work_wide * wide_q_tokens(hg, wide_rows) * 4.0 * s.num_q_heads * s.head_dim;
    const int waves = opt.narrow_waves > 0 ? opt.narrow_waves : narrow_waves(s.num_kv_heads, s.head_dim);
    // Where one launch can hold both kinds of workgroup (the shapes that kernel is
    // built for) a mixed batch of any size runs that way: it costs no packet, and a
    // small batch saves a whole kernel's latency (4 sequences: 20 -> 14 us; the mixed
    // recipe at 1/16 of its size: 38 -> 21 us, at 1/4: 63 -> 51 us).  As two kernels on
    // two streams only when both parts repay the event packets.
    const bool one_launch_shape = !s.kv_merged && (s.kv_fp8 ? s.head_dim == 128 : s.head_dim <= 128) &&
                                  wide_rows == kWideRows && (waves == 1 || waves == 2 || waves == 4);
    if (any_narrow && any_wide && opt.mixed_overlap != 1)
        concurrent = opt.mixed_overlap >= 2 || one_launch_shape || (narrow_bytes >= 128e6 && wide_flops >= 2e10);
    // rough GPU time of the call: the narrow part at 6 TB/s, the wide part at 1 PFLOP/s
    plan.est_gpu_us = narrow_bytes / 6e6 + wide_flops / 1e9;

    const int ny = s.num_kv_heads / waves;
    const int lds_per_wg = waves * narrow_lds_per_wave(s.head_dim); // the same with the 8-bit cache: half the row, twice the stages
    // Four resident waves (one 64 KB workgroup at head_dim 128) per CU already
    // stream at the full HBM rate; more only hold LDS that a wide workgroup of a
    // mixed batch can use, and cut sequences into more pieces.
    // (The 8-bit cache has twice the positions, hence twice the arithmetic, per
    // byte: eight waves per CU there, measured 6 % faster than four, unless a wide
    // workgroup is to fit beside them.)
    // (head_dim 64 has half the bytes per wave in flight: eight waves there too, 200 -> 195 us
    // on 256 sequences of 512-4096 positions)
    // (Both only on a batch large enough to keep that many workgroups busy, about 200
    // MB of K/V: below, twice the bins mean sequences cut in pieces and a combine
    // pass that a short call cannot repay.  128 sequences of 512 positions: head_dim
    // 64 28 against 32 us, 8-bit cache 35 against 39 us.)
    const int waves_per_cu = ((s.kv_fp8 || s.head_dim == 64) && !concurrent && narrow_bytes >= 192e6)
                                 ? 2 * kNarrowWavesPerCu
                                 : kNarrowWavesPerCu;
    const int wgs_per_cu = std::max(1, std::min(kLdsBytesPerCu / lds_per_wg, waves_per_cu / waves));
    const int64_t slots = (int64_t)cus * wgs_per_cu;
    const int oversub = opt.units_per_cu > 0 ? opt.units_per_cu : 1;
    const int64_t want_bins = std::max<int64_t>(1, ceil_div(slots * oversub, ny));
    const int64_t min_bin = 8; // 128 KV positions: below that a bin is not worth a workgroup
    int64_t per_bin = std::max<int64_t>(min_bin, ceil_div(total_tiles, want_bins));
    const int64_t max_piece = opt.kv_chunk > 0 ? ceil_div(opt.kv_chunk, kNarrowKvTile) : ((int64_t)1 << 40);

    // Wide tiles are cut into KV ranges only when there is less than one workgroup
    // per CU and the ranges stay long: a cut tile writes its rows as fp32 partials
    // (twice the bytes of the output, per piece) and adds the combine pass, which
    // costs more than an idle half of the chip gains on anything short (one
    // 2048-token prefill: 73 us cut into 4, 54 us whole; 1024 tokens: 32 / 29 us).
    // What gains is a long context under few query tiles, e.g. a 512-token chunk on
    // 8 K-32 K of context.  Beside the narrow workgroups of a mixed batch the wide
    // part has one slot per CU and usually ends under the narrow part's time (128
    // decode + 4 chunks at Hkv 8: 498 us with more cuts, 438 without); it is cut
    // there only when its longest item alone outlasts both the narrow part and the
    // wide part's own share per slot, i.e. when a few long items are the tail of the
    // call (the same batch at Hq 16 / Hkv 2: 238 us whole, 160-169 us cut).
    int64_t chunk_w;
    if (opt.wide_kv_chunk > 0) {
        chunk_w = round_up(opt.wide_kv_chunk, kWideKvTile);
    } else if (concurrent && wide_tiles * s.num_kv_heads >= (int64_t)cus) {
        // in K/V tiles of the wide kernel: its share per slot, the narrow part's
        // duration (6 TB/s) at about 2 us per wide tile beside it, the longest item
        const double per_slot = (double)work_wide / kWideKvTile * s.num_kv_heads / cus;
        const double narrow_tiles = narrow_bytes / 6e6 / 2.0;
        const double target = std::max(per_slot, narrow_tiles);
        const double longest = (double)longest_wide / kWideKvTile;
        chunk_w = longest > 1.25 * target
                      ? round_up(std::max<int64_t>(1024, (int64_t)(0.75 * target * kWideKvTile)), kWideKvTile)
                      : (int64_t)1 << 30;
    } else {
        // Alone, the wide kernel has two slots per CU with 128-row tiles and one with
        // 256-row tiles.  Between one workgroup per CU and one per slot only long
        // items are cut (8 K positions and more on average: four 256-token chunks on
        // 16 K of context 352 -> 296 us, one 1024-token chunk 364 -> 342 us); shorter
        // ones lose more to the partials than the idle slots cost (two 512-token
        // chunks on 4 K: 103 us whole, 108 us cut).
        const int64_t n_wg = wide_tiles * s.num_kv_heads;
        const int64_t slots = (int64_t)cus * ((concurrent || wide_rows == 256) ? 1 : 2);
        const bool long_items = wide_tiles > 0 && work_wide >= wide_tiles * 8192;
        if (n_wg >= slots || (n_wg >= (int64_t)cus && !long_items))
            chunk_w = (int64_t)1 << 30;
        else
            chunk_w = round_up(
                std::max<int64_t>(concurrent ? 512 : 1024, ceil_div(work_wide * s.num_kv_heads, (int64_t)cus * (concurrent ? 1 : 2))),
                kWideKvTile);
    }

    for (int attempt = 0; attempt < 32; ++attempt) {
        plan.narrow.clear();
        plan.wide.clear();
        plan.items.clear();
        plan.bins.clear();
        int64_t cursor = 0;
        int32_t max_splits = 0;
        int64_t fill = 0;
        plan.bins.push_back(0);
        for (const Tile& t : tiles) {
            if (t.wide) {
                emit_units(t, chunk_w, kWideKvTile, s.num_q_heads, cursor, plan.wide, plan.items, max_splits);
                continue;
            }
            const int64_t w = ceil_div(t.kv_hi, kNarrowKvTile);
            const size_t first = plan.narrow.size();
            int64_t done = 0;
            while (done < w) {
                if (fill >= per_bin) {
                    plan.bins.push_back((int32_t)plan.narrow.size());
                    fill = 0;
                }
                int64_t take = std::min(std::min(w - done, per_bin - fill), max_piece);
                // do not leave a sliver of the tile behind
                if (w - done - take > 0 && w - done - take < 2 && take + (w - done - take) <= max_piece)
                    take = w - done;
                rpa_work_unit u{};
                u.seq = t.seq;
                u.q_start = t.seq_q0 + t.q_pos0;
                u.q_pos0 = t.q_pos0;
                u.n_q = t.n_q;
                u.kv_begin = (int32_t)(done * kNarrowKvTile);
                u.kv_end = (int32_t)std::min<int64_t>((done + take) * kNarrowKvTile, t.kv_hi);
                u.ctx = t.ctx;
                u.seq_q0 = t.seq_q0;
                u.part_row = -1;
                u.flags = 0;
                u.bin = (int32_t)plan.bins.size() - 1;
                plan.narrow.push_back(u);
                done += take;
                fill += take;
            }
            const int64_t n_s = (int64_t)(plan.narrow.size() - first);
            plan.narrow.back().flags |= 1; // the piece that ends the tile writes its new K/V
            max_splits = std::max<int32_t>(max_splits, (int32_t)n_s);
            if (n_s > 1) {
                const int32_t rows = t.n_q * s.num_q_heads;
                const int32_t base = (int32_t)cursor;
                cursor += n_s * rows;
                plan.items.push_back(rpa_combine_item{base, (int32_t)n_s, rows, t.seq_q0 + t.q_pos0});
                for (int64_t k = 0; k < n_s; ++k) plan.narrow[first + k].part_row = (int32_t)(base + k * rows);
            }
        }
        plan.bins.push_back((int32_t)plan.narrow.size());
        if (plan.narrow.empty()) plan.bins.assign(1, 0);
        plan.stats.partial_rows = cursor;
        plan.stats.max_splits = max_splits;
        if (cursor <= partial_row_cap) break;
        if (opt.kv_chunk > 0 || opt.wide_kv_chunk > 0 || attempt == 31) {
            snprintf(buf, sizeof buf, "split partials need %lld rows, workspace holds %lld", (long long)cursor,
                     (long long)partial_row_cap);
            err = buf;
            return RPA_ERR_WORKSPACE;
        }
        per_bin *= 2;
        if (chunk_w < ((int64_t)1 << 30)) chunk_w *= 2;
    }

    // Wide units longest first: the hardware dispatches workgroups in index order,
    // so the short units fill the gaps at the end.  Where the launch is the
    // persistent one (256-row tiles over a bf16 cache in separate pools, short
    // items, nothing narrow beside them) the workgroups walk a fixed schedule with
    // no tail to fill, and the units go by sequence instead, so that the tiles of a
    // sequence run at about the same time and share its K/V in L2 (8 x 2048: HBM
    // traffic 1.78 -> 1.0 x algorithmic, kernel 293 -> 288 us; 16 x 1024: 178 -> 167
    // us).  One workgroup per item by sequence is slower (head_dim 256, 8 x 2048: 775
    // against 733 us; 8-bit cache: 349 against 339 us): the last sequence's long
    // tiles come last.
    auto span = [](const rpa_work_unit& u) { return (int64_t)(u.kv_end - u.kv_begin) * u.n_q; };
    // (with KV heads in multiples of 8 only: there an XCD serves one head of the
    // sequences in flight; Hq 8 / Hkv 1, 8 x 2048: 82 us longest first, 88 us by sequence)
    // (and with sequences of about one length only: the rounds of the fixed schedule
    // pair long with short items of the list as sorted, which ragged sequences taken
    // one after the other are not; 16 prefills of 64-4096 tokens: 917 us longest
    // first, 983 us by sequence)
    int64_t q_min = INT64_MAX, q_max = 0;
    for (const rpa_work_unit& wu : plan.wide) {
        const int64_t lq = (int64_t)cu[wu.seq + 1] - cu[wu.seq];
        q_min = std::min(q_min, lq);
        q_max = std::max(q_max, lq);
    }
    const bool persistent = !any_narrow && wide_rows == 256 && !s.kv_fp8 && !s.kv_merged && s.head_dim <= 128 &&
                            s.num_kv_heads % 8 == 0 && opt.wide_persistent != 1 && plan.wide_persistent_pays() &&
                            2 * q_max <= 3 * q_min;
    const int order = opt.wide_order != 0 ? opt.wide_order : (persistent ? 2 : 1);
    if (order != 2) {
        std::stable_sort(plan.wide.begin(), plan.wide.end(),
                         [&](const rpa_work_unit& a, const rpa_work_unit& b) { return span(a) > span(b); });
    } else {
        // Sequence-major: the tiles of one sequence run at about the same time, so
        // its K/V stay in L2 while they are re-read; heaviest sequence first and,
        // inside a sequence, longest tile first.
        std::vector<int64_t> seq_work(n, 0);
        for (const rpa_work_unit& u : plan.wide) seq_work[u.seq] += span(u);
        std::stable_sort(plan.wide.begin(), plan.wide.end(), [&](const rpa_work_unit& a, const rpa_work_unit& b) {
            if (a.seq != b.seq)
                return seq_work[a.seq] != seq_work[b.seq] ? seq_work[a.seq] > seq_work[b.seq] : a.seq < b.seq;
            return span(a) > span(b);
        });
    }

    plan.stats.concurrent = concurrent;
    plan.stats.num_narrow_bins = (int32_t)plan.bins.size() - 1;
    plan.stats.narrow_waves = waves;
    plan.stats.wide_rows = wide_rows;
    plan.stats.kv_chunk = (int32_t)std::min<int64_t>(per_bin * kNarrowKvTile, INT32_MAX);
    plan.stats.num_narrow_units = (int32_t)plan.narrow.size();
    plan.stats.num_wide_units = (int32_t)plan.wide.size();
    plan.stats.num_combine_items = (int32_t)plan.items.size();
    return RPA_OK;
}

} // namespace rpa
