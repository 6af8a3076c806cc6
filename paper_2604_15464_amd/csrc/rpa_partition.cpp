// Host-side work partitioner and kernel-variant selector.
//
// Algorithm 1 of the paper walks sequences, Q blocks and KV blocks serially on
// one core.  Here the same iteration space is flattened into independent units
// (sequence, Q tile, KV range), one workgroup each, so that 256 compute units
// stay busy: a tile whose KV range is long is cut into several ranges whose
// partial softmax states are merged afterwards.  The regime split of Sec. 3.4
// (decode-only / prefill-only / mixed) becomes a per-sequence choice between
// the narrow and the wide kernel.
#include <algorithm>
#include <cstdio>

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
    if (s.head_dim != 64 && s.head_dim != 128) {
        snprintf(buf, sizeof buf, "head_dim %d unsupported (64 or 128)", s.head_dim);
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
    if ((int64_t)s.num_pages * s.page_size * s.num_kv_heads * s.head_dim >= ((int64_t)1 << 40)) {
        err = "page pool too large";
        return RPA_ERR_UNSUPPORTED;
    }
    return RPA_OK;
}

namespace {

struct Tile {
    int32_t seq, q_pos0, n_q, kv_hi, ctx, seq_q0;
    bool wide;
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
        u.flags = (s == n_s - 1 ? 1 : 0) | (t.wide ? 2 : 0);
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
        opt.wide_kv_chunk < 0) {
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
    const int64_t narrow_max_q = 2 * (int64_t)tq_narrow; // up to two narrow tiles
    bool any_narrow = false, any_wide = false;
    std::vector<Tile> tiles;
    int64_t work_narrow = 0, work_wide = 0, wide_tiles = 0;
    for (int32_t r = 0; r < n; ++r) {
        const int32_t lq = cu[r + 1] - cu[r];
        if (lq == 0) continue;
        bool wide;
        switch (opt.variant) {
        case RPA_VARIANT_DECODE: wide = false; break;
        case RPA_VARIANT_PREFILL: wide = true; break;
        default: wide = lq > narrow_max_q; break;
        }
        (wide ? any_wide : any_narrow) = true;
        const int32_t ctx = kv[r] - lq;
        const int32_t tq = wide ? wide_q_tokens(hg) : tq_narrow;
        for (int32_t i0 = 0; i0 < lq; i0 += tq) {
            Tile t{r, i0, std::min(tq, lq - i0), 0, ctx, cu[r], wide};
            t.kv_hi = ctx + i0 + t.n_q;
            tiles.push_back(t);
            if (wide) {
                work_wide += t.kv_hi;
                ++wide_tiles;
            } else {
                work_narrow += t.kv_hi;
            }
        }
    }
    plan.stats.variant = any_wide ? (any_narrow ? RPA_VARIANT_MIXED : RPA_VARIANT_PREFILL) : RPA_VARIANT_DECODE;

    // ---- KV range per unit ------------------------------------------------
    // Narrow units are bandwidth-bound: equal KV bytes per unit, several units
    // per compute unit so that the tail is short.  Wide units are only split
    // when there are too few tiles to occupy the chip.
    const int cus = std::max(1, num_cus);
    int64_t chunk_n = opt.kv_chunk > 0 ? round_up(opt.kv_chunk, kNarrowKvTile)
                                       : round_up(std::max<int64_t>(256, ceil_div(work_narrow, (int64_t)cus * 6)),
                                                  kNarrowKvTile);
    int64_t chunk_w;
    if (opt.wide_kv_chunk > 0) {
        chunk_w = round_up(opt.wide_kv_chunk, kWideKvTile);
    } else if (wide_tiles * s.num_kv_heads >= (int64_t)cus * 4) {
        chunk_w = (int64_t)1 << 30;
    } else {
        chunk_w = round_up(std::max<int64_t>(512, ceil_div(work_wide * s.num_kv_heads, (int64_t)cus * 4)),
                           kWideKvTile);
    }

    for (int attempt = 0; attempt < 32; ++attempt) {
        plan.narrow.clear();
        plan.wide.clear();
        plan.items.clear();
        int64_t cursor = 0;
        int32_t max_splits = 0;
        for (const Tile& t : tiles) {
            if (t.wide)
                emit_units(t, chunk_w, kWideKvTile, s.num_q_heads, cursor, plan.wide, plan.items, max_splits);
            else
                emit_units(t, chunk_n, kNarrowKvTile, s.num_q_heads, cursor, plan.narrow, plan.items, max_splits);
        }
        plan.stats.partial_rows = cursor;
        plan.stats.max_splits = max_splits;
        if (cursor <= partial_row_cap) break;
        if (opt.kv_chunk > 0 || opt.wide_kv_chunk > 0 || attempt == 31) {
            snprintf(buf, sizeof buf, "split partials need %lld rows, workspace holds %lld", (long long)cursor,
                     (long long)partial_row_cap);
            err = buf;
            return RPA_ERR_WORKSPACE;
        }
        chunk_n *= 2;
        if (chunk_w < ((int64_t)1 << 30)) chunk_w *= 2;
    }

    // Longest first: the hardware dispatches workgroups in index order, so the
    // short units fill the gaps at the end.
    auto span = [](const rpa_work_unit& u) { return (int64_t)(u.kv_end - u.kv_begin) * u.n_q; };
    std::stable_sort(plan.narrow.begin(), plan.narrow.end(),
                     [&](const rpa_work_unit& a, const rpa_work_unit& b) { return span(a) > span(b); });
    std::stable_sort(plan.wide.begin(), plan.wide.end(),
                     [&](const rpa_work_unit& a, const rpa_work_unit& b) { return span(a) > span(b); });

    plan.stats.num_narrow_units = (int32_t)plan.narrow.size();
    plan.stats.num_wide_units = (int32_t)plan.wide.size();
    plan.stats.num_combine_items = (int32_t)plan.items.size();
    plan.stats.kv_chunk = (int32_t)std::min<int64_t>(chunk_n, INT32_MAX);
    return RPA_OK;
}

} // namespace rpa
