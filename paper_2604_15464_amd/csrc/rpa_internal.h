// Internal declarations shared by the host side and the kernel launchers.
#pragma once

#include <stdint.h>

#include <string>
#include <vector>

#include "rpa.h"

namespace rpa {

// Tile geometry the kernels are compiled for.
constexpr int kNarrowRows = 16;   // query rows (tokens x heads of one group) per narrow tile
constexpr int kNarrowKvTile = 16; // KV positions per narrow pipeline stage
constexpr int kWideRows = 128;    // default query rows per wide tile = (128 / h_g) tokens x h_g heads
constexpr int kWideKvTile = 64;   // KV positions per wide pipeline stage
constexpr int kMaxWaves = 8;      // waves per narrow workgroup (one KV head each)
constexpr int kNarrowWavesPerCu = 4; // resident narrow waves per CU: enough to saturate HBM (measured), leaves LDS for a wide workgroup
constexpr int kNarrowStages = 2;   // LDS ring depth of a narrow wave (twice that with the 8-bit cache: same bytes)
constexpr int kWideStages = 3;     // LDS ring depth of a 256-row wide workgroup
constexpr int kWideStagesHalf = 2; // ... of a 128-row one (64 KB: two workgroups per CU)
constexpr int kLdsBytesPerCu = 160 * 1024;

struct Plan {
    std::vector<rpa_work_unit> narrow; // grouped by bin
    std::vector<int32_t> bins;         // bins[b] .. bins[b+1]: the narrow units of workgroup b
    std::vector<rpa_work_unit> wide;   // launch order
    std::vector<rpa_combine_item> items;
    rpa_plan_stats stats{};
    double est_gpu_us = 0; // rough GPU time of the call (narrow bytes at 6 TB/s + wide FLOPs at 1 PFLOP/s)
    // Wide launch form: persistent workgroups pay where items are short (the edges of
    // neighbouring items overlap: config 3, 16 tiles per item on average, -2..4 %);
    // where items are long the walk itself costs more than the edges it hides
    // (one sequence of 16 K-32 K tokens: +1.5 %), and one workgroup per item runs.
    bool wide_persistent_pays() const {
        int64_t tiles = 0;
        for (const rpa_work_unit& u : wide) tiles += (u.kv_end - u.kv_begin + kWideKvTile - 1) / kWideKvTile;
        return !wide.empty() && tiles < (int64_t)64 * (int64_t)wide.size();
    }
};

// Validates shape; returns RPA_OK or an error with a message.
int check_shape(const rpa_shape& s, std::string& err);

// Regime of a batch from its query lengths alone (what AUTO would report):
// DECODE if no sequence is long enough for the wide kernel, PREFILL if all
// non-empty ones are, else MIXED.  Lengths are not validated here.
int classify_batch(const rpa_shape& s, const int32_t* cu_q_lens, int32_t num_seqs);

// Validates the lengths and builds the work partition.
int build_plan(const rpa_shape& s, const int32_t* cu_q_lens, const int32_t* kv_lens,
               int32_t num_seqs, const rpa_options& opt, int num_cus, int64_t partial_row_cap,
               Plan& plan, std::string& err);

// Number of narrow query tokens per tile for a head-group size, or 0 if unsupported.
inline int narrow_q_tokens(int hg) { return (hg >= 1 && hg <= kNarrowRows && kNarrowRows % hg == 0) ? kNarrowRows / hg : 0; }

// Query tokens per wide tile.
inline int wide_q_tokens(int hg, int rows) { return rows / hg; }

// LDS bytes of one narrow wave: ring of stages x (K tile + V tile), then the
// staging area of a unit's Q rows (16 rows of head_dim bf16).
inline int narrow_lds_per_wave(int head_dim) {
    return kNarrowStages * 2 * kNarrowKvTile * head_dim * 2 + kNarrowRows * head_dim * 2;
}

// Default waves per narrow workgroup: the largest divisor of num_kv_heads not
// above 4 (two workgroups of 64 KB LDS per compute unit at head_dim 128, one
// of 128 KB at head_dim 256).
inline int narrow_waves(int hkv, int head_dim) {
    int w = 1;
    for (int d = 1; d <= 4; ++d)
        if (hkv % d == 0 && d * narrow_lds_per_wave(head_dim) <= kLdsBytesPerCu) w = d;
    return w;
}

// Launch-shape options the kernels have no build for at this shape: a narrow
// workgroup whose rings exceed the LDS, 256-row wide tiles at head_dim 256.
inline bool options_fit_shape(const rpa_shape& s, const rpa_options& o) {
    if (o.narrow_waves > 0 && o.narrow_waves * narrow_lds_per_wave(s.head_dim) > kLdsBytesPerCu) return false;
    if (s.head_dim > 128 && o.wide_rows == 256) return false;
    return true;
}

struct KernelArgs {
    const uint16_t* q;
    const uint16_t* k_new;
    const uint16_t* v_new;
    uint16_t* k_pages;
    uint16_t* v_pages;
    uint16_t* out;
    const int32_t* page_table;
    const rpa_work_unit* units;
    const int32_t* bins; // narrow kernel: unit range of each workgroup
    float* part_o;  // [rows, D] un-normalised partial outputs
    float* part_ml; // [rows, 2] running max (log2 domain) and running sum
    int32_t num_q_heads, num_kv_heads, hg, head_dim;
    int32_t page_size_log2, max_pages_per_seq, num_pages;
    int32_t wide_tq_log2; // log2 of the wide tile's token count
    float scale_log2; // sm_scale * log2(e)
    int32_t ablate;   // measurement switches (rpa_options.ablate)
    int32_t causal;   // 0: no mask beyond the end of the sequence
    int32_t kv_fp8;   // 1: pools and k_new / v_new (here: the quantised staging copy) hold E4M3 bytes
    float out_scale;  // V scale of the 8-bit cache, else 1
    int32_t kv_merged; // 1: k_pages is one pool [num_pages, page_size, Hkv, 2, D] with K and V side by side
    int32_t num_wide_items;     // wide kernel: (unit, KV head) pairs of the launch
    const rpa_work_unit* wide_units; // mixed-batch kernel: the wide unit list (units / bins are the narrow one)
    int32_t mixed_narrow_bins;       // ... its narrow bins, waves per narrow task (one bin, that many KV heads),
    int32_t mixed_narrow_waves;      //     narrow workgroups (four waves: 4 / waves tasks each) and wide workgroups
    int32_t mixed_narrow_wgs;
    int32_t mixed_wide_wgs;
    int32_t wide_persist_grid;  // > 0: workgroups of the persistent wide kernel (one per CU), which walk the items
};

// Launchers (rpa_kernels.hip).  Return a hipError_t value as int.  `ev` is either
// null or two hipEvent_t that receive the kernel's own start and stop times
// (attached to the dispatch, no extra queue packets).
int launch_narrow(const KernelArgs& a, int num_bins, int waves, void* stream, void** ev);
bool mixed_launch_built(const KernelArgs& a, int narrow_waves);
int launch_mixed(const KernelArgs& a, int num_bins, int narrow_waves, int num_wide_units, void* stream, void** ev);
int launch_wide(const KernelArgs& a, int num_units, void* stream, void** ev);
int launch_combine(const rpa_combine_item* items, int num_items, const float* part_o,
                   const float* part_ml, uint16_t* out, int num_q_heads, int head_dim, int max_rows,
                   void* stream, void** ev);
int launch_copy(void* dst, const void* src, size_t n16, int num_cus, void* stream, void** ev);
int launch_mfma(int steps, int num_cus, void* stream, void** ev);
// new K/V rows (bf16, `elems` elements each, a multiple of 8) -> E4M3 bytes of x * inv_scale
int launch_quantize(const void* k_new, const void* v_new, void* k8, void* v8, size_t elems, float inv_k, float inv_v,
                    int num_cus, void* stream);
int kernels_init(int device, std::string& err);

} // namespace rpa
