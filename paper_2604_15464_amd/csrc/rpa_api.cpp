// C ABI of the library: context, validation, per-call planning and launches.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "rpa_internal.h"

using namespace rpa;

namespace {

constexpr int kRing = 8;  // staging slots: the host may run this many calls ahead of the GPU
constexpr double kInPlaceListBelowUs = 30.0; // calls estimated shorter than this read their work list from host memory
constexpr int kGroup = 4; // calls that share one completion event (an event record is a stream
                          // packet of its own and costs the GPU about 5 us of idle time)

thread_local std::string g_err; // errors without a context

struct Staging {
    void* host = nullptr;        // pinned
    void* dev = nullptr;         // device copy of the same blob
    hipEvent_t done = nullptr;   // recorded on the caller's stream after a group of calls
    hipEvent_t* cover = nullptr; // the recorded event that tells that the kernels reading `dev` finished
    hipEvent_t fork = nullptr;   // caller's stream has reached this call (side stream waits for it)
    hipEvent_t join = nullptr;   // side stream's kernel finished (caller's stream waits for it)
    hipEvent_t uploaded = nullptr; // the work list has reached `dev` (stream-ordered upload only)
    bool used = false;
};

} // namespace

constexpr int kProfCalls = 1024;

struct ProfEvents {
    hipEvent_t ev[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr}; // start/stop of narrow, wide, combine
    bool narrow = false, wide = false, combine = false;
};

struct rpa_ctx {
    bool prof_on = false;
    std::vector<ProfEvents> prof;
    int prof_count = 0;
    rpa_shape shape{};
    rpa_options opt{};             // set of rpa_set_options()
    rpa_options regime_opt[4]{};   // per-regime sets, indexed by rpa_variant
    bool regime_set[4] = {false, false, false, false};
    int device = 0;
    int num_cus = 0;
    int max_units = 0;
    int max_items = 0;
    int64_t partial_row_cap = 0;
    size_t blob_bytes = 0;
    Staging ring[kRing];
    int ring_pos = 0;
    int pending[kGroup];          // slots of the calls since the last completion event
    int num_pending = 0;
    hipStream_t last_stream = nullptr; // stream of those calls
    hipStream_t upload = nullptr; // work lists are uploaded here, ahead of the caller's stream
    hipStream_t side = nullptr;   // the wide kernel of a mixed batch runs here, beside the narrow one
    float* part_o = nullptr;
    float* part_ml = nullptr;
    void* new8_k = nullptr; // 8-bit cache: quantised copy of this call's k_new / v_new rows
    void* new8_v = nullptr;
    int64_t workspace_bytes = 0;
    Plan plan;
    rpa_plan_stats last{};
    std::string err;
};

static int fail(rpa_ctx* c, int code, const std::string& msg) {
    if (c)
        c->err = msg;
    else
        g_err = msg;
    return code;
}

static int hip_fail(rpa_ctx* c, const char* what, hipError_t e) {
    return fail(c, RPA_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

extern "C" int rpa_create(rpa_ctx** out, const rpa_shape* shape, int device) {
    if (!out || !shape) return fail(nullptr, RPA_ERR_INVALID_ARG, "rpa_create: null argument");
    std::string msg;
    int rc = check_shape(*shape, msg);
    if (rc != RPA_OK) return fail(nullptr, rc, msg);
    hipError_t e = hipSetDevice(device);
    if (e != hipSuccess) return hip_fail(nullptr, "hipSetDevice", e);
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, device);
    if (e != hipSuccess) return hip_fail(nullptr, "hipGetDeviceProperties", e);
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return fail(nullptr, RPA_ERR_UNSUPPORTED, std::string("device is ") + prop.gcnArchName + ", kernels are gfx950 only");

    rpa_ctx* c = new (std::nothrow) rpa_ctx();
    if (!c) return fail(nullptr, RPA_ERR_HIP, "out of host memory");
    c->shape = *shape;
    c->device = device;
    c->num_cus = prop.multiProcessorCount;
    // Units: every query tile once, plus the extra ranges of split tiles
    // (bounded by the per-CU oversubscription of the partitioner).
    const int hg = shape->num_q_heads / shape->num_kv_heads;
    const int64_t tiles = (int64_t)shape->max_tokens / 1 + shape->max_seqs;
    (void)hg;
    c->max_units = (int)std::min<int64_t>(tiles + 64 * (int64_t)c->num_cus, 1 << 24);
    c->max_items = c->max_units;
    // Split partials: a narrow unit holds 16 rows per KV head, a wide unit 256;
    // the partitioner keeps a handful of units per compute unit.
    c->partial_row_cap = std::min<int64_t>(
        std::max<int64_t>((int64_t)8 * shape->max_tokens * shape->num_q_heads,
                          (int64_t)12 * c->num_cus * kNarrowRows * shape->num_kv_heads),
        (int64_t)1 << 20);
    c->blob_bytes = (size_t)c->max_units * (sizeof(rpa_work_unit) + sizeof(rpa_combine_item) + sizeof(int32_t)) + 64;

    auto cleanup = [&](const char* what, hipError_t err) {
        int r = hip_fail(nullptr, what, err);
        rpa_destroy(c);
        return r;
    };
    for (int i = 0; i < kRing; ++i) {
        e = hipHostMalloc(&c->ring[i].host, c->blob_bytes, hipHostMallocDefault);
        if (e != hipSuccess) return cleanup("hipHostMalloc", e);
        e = hipMalloc(&c->ring[i].dev, c->blob_bytes);
        if (e != hipSuccess) return cleanup("hipMalloc", e);
        e = hipEventCreateWithFlags(&c->ring[i].done, hipEventDisableTiming);
        if (e != hipSuccess) return cleanup("hipEventCreate", e);
        e = hipEventCreateWithFlags(&c->ring[i].fork, hipEventDisableTiming);
        if (e != hipSuccess) return cleanup("hipEventCreate", e);
        e = hipEventCreateWithFlags(&c->ring[i].join, hipEventDisableTiming);
        if (e != hipSuccess) return cleanup("hipEventCreate", e);
        e = hipEventCreateWithFlags(&c->ring[i].uploaded, hipEventDisableTiming);
        if (e != hipSuccess) return cleanup("hipEventCreate", e);
        c->workspace_bytes += (int64_t)c->blob_bytes;
    }
    e = hipStreamCreateWithFlags(&c->upload, hipStreamNonBlocking);
    if (e != hipSuccess) return cleanup("hipStreamCreate", e);
    e = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking);
    if (e != hipSuccess) return cleanup("hipStreamCreate", e);
    const size_t po = (size_t)c->partial_row_cap * shape->head_dim * sizeof(float);
    const size_t pml = (size_t)c->partial_row_cap * 2 * sizeof(float);
    e = hipMalloc((void**)&c->part_o, po);
    if (e != hipSuccess) return cleanup("hipMalloc", e);
    e = hipMalloc((void**)&c->part_ml, pml);
    if (e != hipSuccess) return cleanup("hipMalloc", e);
    c->workspace_bytes += (int64_t)(po + pml);
    if (shape->kv_fp8) {
        const size_t nb = (size_t)shape->max_tokens * shape->num_kv_heads * shape->head_dim;
        e = hipMalloc(&c->new8_k, nb);
        if (e != hipSuccess) return cleanup("hipMalloc", e);
        e = hipMalloc(&c->new8_v, nb);
        if (e != hipSuccess) return cleanup("hipMalloc", e);
        c->workspace_bytes += (int64_t)(2 * nb);
    }
    if (kernels_init(device, msg) != 0) {
        rpa_destroy(c);
        return fail(nullptr, RPA_ERR_HIP, msg);
    }
    *out = c;
    return RPA_OK;
}

extern "C" void rpa_destroy(rpa_ctx* c) {
    if (!c) return;
    // kernels of the last calls may still read the work lists (some from the pinned
    // host slots) and the partials
    int prev = -1;
    if (hipGetDevice(&prev) == hipSuccess && prev != c->device) (void)hipSetDevice(c->device);
    (void)hipDeviceSynchronize();
    for (int i = 0; i < kRing; ++i) {
        if (c->ring[i].done) (void)hipEventDestroy(c->ring[i].done);
        if (c->ring[i].fork) (void)hipEventDestroy(c->ring[i].fork);
        if (c->ring[i].join) (void)hipEventDestroy(c->ring[i].join);
        if (c->ring[i].uploaded) (void)hipEventDestroy(c->ring[i].uploaded);
        if (c->ring[i].host) (void)hipHostFree(c->ring[i].host);
        if (c->ring[i].dev) (void)hipFree(c->ring[i].dev);
    }
    if (c->upload) (void)hipStreamDestroy(c->upload);
    if (c->side) (void)hipStreamDestroy(c->side);
    if (c->part_o) (void)hipFree(c->part_o);
    if (c->part_ml) (void)hipFree(c->part_ml);
    if (c->new8_k) (void)hipFree(c->new8_k);
    if (c->new8_v) (void)hipFree(c->new8_v);
    for (auto& p : c->prof)
        for (auto& e : p.ev)
            if (e) (void)hipEventDestroy(e);
    if (prev >= 0 && prev != c->device) (void)hipSetDevice(prev);
    delete c;
}

extern "C" const char* rpa_last_error(const rpa_ctx* c) { return c ? c->err.c_str() : g_err.c_str(); }

extern "C" int rpa_plan_info(const rpa_ctx* c, rpa_plan_stats* out) {
    if (!c || !out) return RPA_ERR_INVALID_ARG;
    *out = c->last;
    out->workspace_bytes = c->workspace_bytes;
    return RPA_OK;
}

extern "C" int rpa_set_options(rpa_ctx* c, const rpa_options* opt) {
    if (!c) return RPA_ERR_INVALID_ARG;
    rpa_options o{};
    if (opt) o = *opt;
    if (o.variant < RPA_VARIANT_AUTO || o.variant > RPA_VARIANT_MIXED || o.kv_chunk < 0 || o.wide_kv_chunk < 0 ||
        o.units_per_cu < 0 || o.narrow_waves < 0 || o.narrow_waves > kMaxWaves ||
        (o.narrow_waves > 0 && c->shape.num_kv_heads % o.narrow_waves != 0) ||
        (o.wide_rows != 0 && o.wide_rows != 128 && o.wide_rows != 256) || o.wide_order < 0 || o.wide_order > 2 ||
        o.mixed_overlap < 0 || o.mixed_overlap > 3 || o.stream_ordered_upload < 0 || o.stream_ordered_upload > 3 ||
        o.wide_persistent < 0 || o.wide_persistent > 1 || !options_fit_shape(c->shape, o))
        return fail(c, RPA_ERR_INVALID_ARG, "rpa_set_options: bad value");
#ifdef RPA_ABLATE
    if (o.ablate & ~(1 | 2 | 4 | 64 | 128 | 256 | 512))
        return fail(c, RPA_ERR_INVALID_ARG, "rpa_set_options: unknown ablation bit");
#else
    if (o.ablate != 0)
        return fail(c, RPA_ERR_UNSUPPORTED,
                    "rpa_set_options: this library is built without the measurement switches (the ablation build has them)");
#endif
    c->opt = o;
    for (bool& b : c->regime_set) b = false;
    return RPA_OK;
}

extern "C" int rpa_set_regime_options(rpa_ctx* c, int32_t regime, const rpa_options* opt) {
    if (!c) return RPA_ERR_INVALID_ARG;
    if (regime < RPA_VARIANT_DECODE || regime > RPA_VARIANT_MIXED)
        return fail(c, RPA_ERR_INVALID_ARG, "rpa_set_regime_options: regime must be decode, prefill or mixed");
    rpa_options o{};
    if (opt) o = *opt;
    if (o.variant != RPA_VARIANT_AUTO && o.variant != regime)
        return fail(c, RPA_ERR_INVALID_ARG, "rpa_set_regime_options: variant must be auto or the regime itself");
    // the same checks as rpa_set_options
    const rpa_options keep = c->opt;
    bool keep_set[4];
    for (int i = 0; i < 4; ++i) keep_set[i] = c->regime_set[i];
    const int rc = rpa_set_options(c, &o);
    c->opt = keep;
    for (int i = 0; i < 4; ++i) c->regime_set[i] = keep_set[i];
    if (rc != RPA_OK) return rc;
    c->regime_opt[regime] = o;
    c->regime_set[regime] = true;
    return RPA_OK;
}

extern "C" int rpa_profile_enable(rpa_ctx* c, int on) {
    if (!c) return RPA_ERR_INVALID_ARG;
    if (on && c->prof.empty()) {
        c->prof.resize(kProfCalls);
        for (auto& p : c->prof)
            for (auto& e : p.ev) {
                hipError_t err = hipEventCreate(&e);
                if (err != hipSuccess) return hip_fail(c, "hipEventCreate", err);
            }
    }
    c->prof_on = on != 0;
    c->prof_count = 0;
    return RPA_OK;
}

extern "C" int rpa_profile_read(rpa_ctx* c, float* narrow_ms, float* wide_ms, float* combine_ms, int32_t* calls) {
    if (!c || !narrow_ms || !wide_ms || !combine_ms || !calls) return RPA_ERR_INVALID_ARG;
    *narrow_ms = *wide_ms = *combine_ms = 0.f;
    *calls = c->prof_count;
    for (int i = 0; i < c->prof_count; ++i) {
        ProfEvents& p = c->prof[i];
        const bool has[3] = {p.narrow, p.wide, p.combine};
        float* dst[3] = {narrow_ms, wide_ms, combine_ms};
        for (int k = 0; k < 3; ++k) {
            if (!has[k]) continue;
            hipError_t e = hipEventSynchronize(p.ev[2 * k + 1]);
            if (e != hipSuccess) return hip_fail(c, "hipEventSynchronize", e);
            float ms = 0.f;
            e = hipEventElapsedTime(&ms, p.ev[2 * k], p.ev[2 * k + 1]);
            if (e != hipSuccess) return hip_fail(c, "hipEventElapsedTime", e);
            *dst[k] += ms;
        }
    }
    c->prof_count = 0;
    return RPA_OK;
}

extern "C" int rpa_copy_probe(rpa_ctx* c, void* dst, const void* src, size_t bytes, void* stream, float* ms) {
    if (!c) return RPA_ERR_INVALID_ARG;
    if (!dst || !src || bytes % 16 != 0 || ((uintptr_t)dst | (uintptr_t)src) % 16 != 0)
        return fail(c, RPA_ERR_INVALID_ARG, "rpa_copy_probe: pointers and size must be multiples of 16");
    const char *d = (const char*)dst, *s = (const char*)src;
    if (d < s + bytes && s < d + bytes) return fail(c, RPA_ERR_INVALID_ARG, "rpa_copy_probe: ranges overlap");
    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, "hipSetDevice", e);
    hipEvent_t ev[2] = {nullptr, nullptr};
    if (ms) {
        for (auto& x : ev) {
            e = hipEventCreate(&x);
            if (e != hipSuccess) {
                if (ev[0]) (void)hipEventDestroy(ev[0]);
                return hip_fail(c, "hipEventCreate", e);
            }
        }
    }
    int rc = launch_copy(dst, src, bytes / 16, c->num_cus, stream, ms ? (void**)ev : nullptr);
    if (rc == 0 && ms) {
        e = hipEventSynchronize(ev[1]);
        if (e == hipSuccess) e = hipEventElapsedTime(ms, ev[0], ev[1]);
        rc = (int)e;
    }
    for (auto& x : ev)
        if (x) (void)hipEventDestroy(x);
    if (rc != 0) return hip_fail(c, "rpa_copy_probe", (hipError_t)rc);
    return RPA_OK;
}

extern "C" int rpa_mfma_probe(rpa_ctx* c, int32_t steps, void* stream, float* ms, double* flops) {
    if (!c) return RPA_ERR_INVALID_ARG;
    if (steps < 1 || steps > (1 << 20)) return fail(c, RPA_ERR_INVALID_ARG, "rpa_mfma_probe: steps must be in [1, 2^20]");
    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, "hipSetDevice", e);
    hipEvent_t ev[2] = {nullptr, nullptr};
    if (ms) {
        for (auto& x : ev) {
            e = hipEventCreate(&x);
            if (e != hipSuccess) {
                if (ev[0]) (void)hipEventDestroy(ev[0]);
                return hip_fail(c, "hipEventCreate", e);
            }
        }
    }
    int rc = launch_mfma(steps, c->num_cus, stream, ms ? (void**)ev : nullptr);
    if (rc == 0 && ms) {
        e = hipEventSynchronize(ev[1]);
        if (e == hipSuccess) e = hipEventElapsedTime(ms, ev[0], ev[1]);
        rc = (int)e;
    }
    for (auto& x : ev)
        if (x) (void)hipEventDestroy(x);
    if (rc != 0) return hip_fail(c, "rpa_mfma_probe", (hipError_t)rc);
    // workgroups x 8 waves x steps x 32 MFMAs of 2 * 32 * 32 * 16 FLOPs
    if (flops) *flops = (double)c->num_cus * 8.0 * (double)steps * 32.0 * 32768.0;
    return RPA_OK;
}

extern "C" int rpa_plan_host(const rpa_shape* shape, const int32_t* cu_q_lens, const int32_t* kv_lens,
                             int32_t num_seqs, const rpa_options* opt, int num_cus, rpa_work_unit* units,
                             int32_t max_units, rpa_combine_item* items, int32_t max_items,
                             rpa_plan_stats* stats) {
    if (!shape || !stats || max_units < 0 || max_items < 0 || (max_units > 0 && !units) || (max_items > 0 && !items))
        return fail(nullptr, RPA_ERR_INVALID_ARG, "rpa_plan_host: bad argument");
    std::string msg;
    int rc = check_shape(*shape, msg);
    if (rc != RPA_OK) return fail(nullptr, rc, msg);
    rpa_options o{};
    if (opt) o = *opt;
    Plan plan;
    rc = build_plan(*shape, cu_q_lens, kv_lens, num_seqs, o, num_cus, (int64_t)1 << 40, plan, msg);
    if (rc != RPA_OK) return fail(nullptr, rc, msg);
    *stats = plan.stats;
    const size_t nu = plan.narrow.size() + plan.wide.size();
    if (nu > (size_t)max_units || plan.items.size() > (size_t)max_items)
        return fail(nullptr, RPA_ERR_WORKSPACE, "rpa_plan_host: output buffers too small");
    if (!plan.narrow.empty()) std::memcpy(units, plan.narrow.data(), plan.narrow.size() * sizeof(rpa_work_unit));
    if (!plan.wide.empty())
        std::memcpy(units + plan.narrow.size(), plan.wide.data(), plan.wide.size() * sizeof(rpa_work_unit));
    if (!plan.items.empty()) std::memcpy(items, plan.items.data(), plan.items.size() * sizeof(rpa_combine_item));
    return RPA_OK;
}

extern "C" int rpa_update_and_attend(rpa_ctx* c, void* out, const void* q, const void* k_new, const void* v_new,
                                     void* k_pages, void* v_pages, const int32_t* page_table,
                                     const int32_t* cu_q_lens, const int32_t* kv_lens, int32_t num_seqs,
                                     float sm_scale, void* stream) {
    if (!c) return RPA_ERR_INVALID_ARG;
    if (num_seqs == 0) {
        c->last = rpa_plan_stats{};
        return RPA_OK;
    }
    if (!out || !q || !k_new || !v_new || !k_pages || (!v_pages && !c->shape.kv_merged) || !page_table)
        return fail(c, RPA_ERR_INVALID_ARG, "rpa_update_and_attend: null tensor pointer");
    const uintptr_t align = (uintptr_t)out | (uintptr_t)q | (uintptr_t)k_new | (uintptr_t)v_new |
                            (uintptr_t)k_pages | (uintptr_t)v_pages;
    if (align & 15) return fail(c, RPA_ERR_INVALID_ARG, "rpa_update_and_attend: tensors must be 16-byte aligned");
    if (!std::isfinite(sm_scale) || !(sm_scale > 0.f))
        return fail(c, RPA_ERR_INVALID_ARG, "rpa_update_and_attend: sm_scale must be finite and positive");

    std::string msg;
    if (num_seqs < 0 || num_seqs > c->shape.max_seqs || !cu_q_lens || !kv_lens)
        return fail(c, num_seqs < 0 || num_seqs > c->shape.max_seqs ? RPA_ERR_BAD_LENGTHS : RPA_ERR_INVALID_ARG,
                    "rpa_update_and_attend: num_seqs outside [0, max_seqs] or a length array is null");
    // the regime's own set of knobs, if one was given (Sec. 3.1.4)
    const int regime = classify_batch(c->shape, cu_q_lens, num_seqs);
    const rpa_options& opt_used = c->regime_set[regime] ? c->regime_opt[regime] : c->opt;
    int rc = build_plan(c->shape, cu_q_lens, kv_lens, num_seqs, opt_used, c->num_cus, c->partial_row_cap, c->plan, msg);
    if (rc != RPA_OK) return fail(c, rc, msg);
    Plan& plan = c->plan;
    const size_t n_narrow = plan.narrow.size(), n_wide = plan.wide.size(), n_items = plan.items.size();
    if (n_narrow + n_wide == 0) {
        c->last = plan.stats;
        return RPA_OK;
    }
    if (n_narrow + n_wide > (size_t)c->max_units || n_items > (size_t)c->max_items)
        return fail(c, RPA_ERR_WORKSPACE, "work list larger than the workspace sized at create");

    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, "hipSetDevice", e);
    hipStream_t st = (hipStream_t)stream;
    // Completion events are shared by groups of kGroup calls on one stream.  A call
    // on another stream closes the group of the calls before it.
    auto close_group = [&](hipStream_t on) -> hipError_t {
        if (c->num_pending == 0) return hipSuccess;
        Staging& last = c->ring[c->pending[c->num_pending - 1]];
        const hipError_t r = hipEventRecord(last.done, on);
        if (r != hipSuccess) return r;
        for (int i = 0; i < c->num_pending; ++i) c->ring[c->pending[i]].cover = &last.done;
        c->num_pending = 0;
        return hipSuccess;
    };
    if (c->num_pending > 0 && st != c->last_stream) {
        e = close_group(c->last_stream);
        if (e != hipSuccess) return hip_fail(c, "hipEventRecord", e);
    }
    // The work list goes up on the library's own stream so that it overlaps the
    // previous call's kernels.  The slot is reused once the kernels of the call
    // that used it kRing calls ago are done: its group's event was recorded at
    // least kRing - kGroup calls ago, so this wait does not stall in steady state.
    Staging& slot = c->ring[c->ring_pos];
    if (slot.used) {
        if (!slot.cover) {
            // only after a call that failed half way (its slot never joined a group)
            e = close_group(c->last_stream);
            if (e != hipSuccess) return hip_fail(c, "hipEventRecord", e);
        }
        e = slot.cover ? hipEventSynchronize(*slot.cover) : hipDeviceSynchronize();
        if (e != hipSuccess) return hip_fail(c, "hipEventSynchronize", e);
        slot.cover = nullptr;
    }
    const int slot_index = c->ring_pos;
    char* h = (char*)slot.host;
    const size_t units_bytes = (n_narrow + n_wide) * sizeof(rpa_work_unit);
    const size_t items_off = (units_bytes + 15) & ~(size_t)15;
    const size_t bins_off = items_off + n_items * sizeof(rpa_combine_item);
    const size_t n_bins = n_narrow ? plan.bins.size() - 1 : 0;
    const size_t total_bytes = bins_off + plan.bins.size() * sizeof(int32_t);
    if (total_bytes > c->blob_bytes) return fail(c, RPA_ERR_WORKSPACE, "work list larger than the workspace sized at create");
    if (n_narrow) std::memcpy(h, plan.narrow.data(), n_narrow * sizeof(rpa_work_unit));
    if (n_wide) std::memcpy(h + n_narrow * sizeof(rpa_work_unit), plan.wide.data(), n_wide * sizeof(rpa_work_unit));
    if (n_items) std::memcpy(h + items_off, plan.items.data(), n_items * sizeof(rpa_combine_item));
    std::memcpy(h + bins_off, plan.bins.data(), plan.bins.size() * sizeof(int32_t));
    // How the list reaches the kernels.  A short call is bound by latency: the copy,
    // the host's wait for it and the launch come one after the other while the GPU
    // idles, so the kernels read the list where the host wrote it (pinned,
    // device-visible host memory; a record is read once per unit, by scalar loads
    // issued ahead of their use): 30 -> 20 us per call on a batch of four short
    // sequences, 27 -> 18 us on one 512-token prefill.  A long call hides the copy
    // behind the previous call's kernels, and reading the records over PCIe would
    // cost its kernels 1-3 us (a 45 us decode batch: +1-2 us): there the list is
    // copied to device memory on the library's stream and the host waits for that
    // small copy (a wait packet on the caller's stream instead costs the GPU about
    // 5 us of idle time per call; stream_ordered_upload = 1 selects it: the host
    // never waits).  The caller's stream is not synchronised in any form.
    const int upload = opt_used.stream_ordered_upload;
    const bool in_place = upload == 2 || (upload == 0 && plan.est_gpu_us < kInPlaceListBelowUs);
    const char* list = (const char*)slot.dev;
    if (in_place) {
        void* mapped = nullptr;
        e = hipHostGetDevicePointer(&mapped, slot.host, 0);
        if (e != hipSuccess) return hip_fail(c, "hipHostGetDevicePointer", e);
        list = (const char*)mapped;
    } else {
        e = hipMemcpyAsync(slot.dev, h, total_bytes, hipMemcpyHostToDevice, c->upload);
        if (e != hipSuccess) return hip_fail(c, "hipMemcpyAsync", e);
        if (upload == 1) {
            e = hipEventRecord(slot.uploaded, c->upload);
            if (e != hipSuccess) return hip_fail(c, "hipEventRecord", e);
            e = hipStreamWaitEvent(st, slot.uploaded, 0);
            if (e != hipSuccess) return hip_fail(c, "hipStreamWaitEvent", e);
        } else {
            e = hipStreamSynchronize(c->upload);
            if (e != hipSuccess) return hip_fail(c, "hipStreamSynchronize", e);
        }
    }
    (void)hipGetLastError(); // a stale error of an earlier HIP call is not a launch failure of this call
    slot.used = true;
    c->ring_pos = (c->ring_pos + 1) % kRing;

    KernelArgs a{};
    a.q = (const uint16_t*)q;
    a.k_new = (const uint16_t*)k_new;
    a.v_new = (const uint16_t*)v_new;
    a.k_pages = (uint16_t*)k_pages;
    a.v_pages = (uint16_t*)v_pages;
    a.out = (uint16_t*)out;
    a.page_table = page_table;
    a.part_o = c->part_o;
    a.part_ml = c->part_ml;
    a.num_q_heads = c->shape.num_q_heads;
    a.num_kv_heads = c->shape.num_kv_heads;
    a.hg = c->shape.num_q_heads / c->shape.num_kv_heads;
    a.head_dim = c->shape.head_dim;
    a.page_size_log2 = __builtin_ctz((unsigned)c->shape.page_size);
    a.max_pages_per_seq = c->shape.max_pages_per_seq;
    a.num_pages = c->shape.num_pages;
    a.wide_tq_log2 = __builtin_ctz((unsigned)wide_q_tokens(a.hg, plan.stats.wide_rows));
    a.scale_log2 = sm_scale * 1.4426950408889634f;
    a.ablate = opt_used.ablate;
    a.causal = c->shape.non_causal ? 0 : 1;
    a.kv_fp8 = c->shape.kv_fp8;
    a.out_scale = 1.f;
    a.kv_merged = c->shape.kv_merged;
    a.wide_persist_grid = (opt_used.wide_persistent == 1 || !plan.wide_persistent_pays()) ? 0 : c->num_cus;
    if (a.kv_fp8) {
        // The new rows are quantised into the staging copy first; from there on the
        // kernels see bytes only.  K's scale folds into the softmax scale, V's is
        // applied to the output rows.
        const size_t elems = (size_t)cu_q_lens[num_seqs] * a.num_kv_heads * a.head_dim;
        const int qrc = launch_quantize(k_new, v_new, c->new8_k, c->new8_v, elems, 1.f / c->shape.k_scale,
                                        1.f / c->shape.v_scale, c->num_cus, stream);
        if (qrc != 0) return hip_fail(c, "quantise kernel launch", (hipError_t)qrc);
        a.k_new = (const uint16_t*)c->new8_k;
        a.v_new = (const uint16_t*)c->new8_v;
        a.scale_log2 *= c->shape.k_scale;
        a.out_scale = c->shape.v_scale;
    }

    const rpa_work_unit* dev_units = (const rpa_work_unit*)list;
    ProfEvents* pe = (c->prof_on && c->prof_count < kProfCalls) ? &c->prof[c->prof_count] : nullptr;
    int hrc;
    a.units = dev_units;
    a.bins = (const int32_t*)(list + bins_off);
    // Mixed batch: the wide kernel goes to the context's side stream, forked here
    // (after the caller's stream has the work list) and joined before the combine.
    // The two kernels touch disjoint query tokens, partial rows and cache slots.
    const bool concurrent = plan.stats.concurrent != 0;
    // one launch with both kinds of workgroup where that kernel is built, else two
    // kernels on two streams
    const bool one_launch = concurrent && opt_used.mixed_overlap != 3 && n_narrow > 0 && n_wide > 0 &&
                            mixed_launch_built(a, plan.stats.narrow_waves);
    if (one_launch) {
        a.wide_units = dev_units + n_narrow;
        hrc = launch_mixed(a, (int)n_bins, plan.stats.narrow_waves, (int)n_wide, stream, pe ? (void**)&pe->ev[0] : nullptr);
        if (hrc != 0) return hip_fail(c, "mixed kernel launch", (hipError_t)hrc);
        plan.stats.concurrent = 2;
    }
    void* wide_stream = stream;
    if (concurrent && !one_launch) {
        e = hipEventRecord(slot.fork, st);
        if (e != hipSuccess) return hip_fail(c, "hipEventRecord", e);
        e = hipStreamWaitEvent(c->side, slot.fork, 0);
        if (e != hipSuccess) return hip_fail(c, "hipStreamWaitEvent", e);
        wide_stream = (void*)c->side;
    }
    if (!one_launch) {
        hrc = launch_narrow(a, (int)n_bins, plan.stats.narrow_waves, stream, pe ? (void**)&pe->ev[0] : nullptr);
        if (hrc != 0) return hip_fail(c, "narrow kernel launch", (hipError_t)hrc);
        a.units = dev_units + n_narrow;
        hrc = launch_wide(a, (int)n_wide, wide_stream, pe ? (void**)&pe->ev[2] : nullptr);
        if (hrc != 0) return hip_fail(c, "wide kernel launch", (hipError_t)hrc);
    }
    if (concurrent && !one_launch) {
        e = hipEventRecord(slot.join, c->side);
        if (e != hipSuccess) return hip_fail(c, "hipEventRecord", e);
        e = hipStreamWaitEvent(st, slot.join, 0);
        if (e != hipSuccess) return hip_fail(c, "hipStreamWaitEvent", e);
    }
    int max_rows = 0;
    for (const rpa_combine_item& it : plan.items) max_rows = std::max(max_rows, (int)it.rows);
    hrc = launch_combine((const rpa_combine_item*)(list + items_off), (int)n_items, c->part_o, c->part_ml,
                         (uint16_t*)out, a.num_q_heads, a.head_dim, max_rows, stream,
                         pe ? (void**)&pe->ev[4] : nullptr);
    if (hrc != 0) return hip_fail(c, "combine kernel launch", (hipError_t)hrc);
    c->pending[c->num_pending++] = slot_index;
    c->last_stream = st;
    if (c->num_pending == kGroup) {
        e = close_group(st);
        if (e != hipSuccess) return hip_fail(c, "hipEventRecord", e);
    }
    if (pe) {
        pe->narrow = n_narrow > 0;
        pe->wide = n_wide > 0 && !one_launch; // the one launch of a mixed batch is timed as the narrow kernel
        pe->combine = n_items > 0;
        ++c->prof_count;
    }
    c->last = plan.stats;
    return RPA_OK;
}
