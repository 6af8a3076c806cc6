// rpa_update_and_attend_noalloc: the hot call for callers that cannot allocate
// (code under stream capture, serving loops and harnesses that forbid
// hipMalloc).  Same host partitioner and the same kernels as
// rpa_update_and_attend; what a context keeps in buffers allocated at
// rpa_create (device work list, split partials) lives here in one file-scope
// device array, and the work list travels to it inside kernel arguments, so no
// staging memory, stream or event is needed either.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <string>

#include "rpa_internal.h"

namespace {

constexpr size_t kListBytes = 64 * 1024;          // work list: units, combine items, bins
constexpr size_t kPartialBytes = 8 * 1024 * 1024; // split partials: (m, l) pairs, then O rows
constexpr size_t kScratchBytes = kListBytes + kPartialBytes;
constexpr int kMaxDevices = 16;

// One copy per GPU the library is loaded on, held until the process ends.  Host
// code must never use this name as an address: the per-device address comes
// from hipGetSymbolAddress (device_state below).
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// A piece of the work list, carried by value in the kernel arguments (the
// runtime copies them at launch, so the host buffer is free again on return).
constexpr int kPokeWords = 960;
struct PokePayload {
    uint32_t w[kPokeWords];
};

__global__ void __launch_bounds__(256) rpa_poke_kernel(PokePayload p, uint32_t* dst, int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) dst[i] = p.w[i];
}

struct DeviceState {
    bool ready = false;
    unsigned char* ptr = nullptr; // this device's copy of `scratch`
    int num_cus = 0;
    rpa::Plan plan;               // host vectors, reused from call to call
    std::string blob;             // host image of the work list
};

DeviceState g_state[kMaxDevices];
thread_local std::string g_noalloc_err;

int fail(int code, const std::string& msg) {
    g_noalloc_err = msg;
    return code;
}

int hip_fail(const char* what, hipError_t e) {
    return fail(RPA_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

// Set-up, once per device, with that device current: the address of this
// device's copy of the array, the CU count, the kernels' LDS attributes.
int device_state(int device, DeviceState** out) {
    if (device < 0 || device >= kMaxDevices) return fail(RPA_ERR_INVALID_ARG, "device index out of range");
    DeviceState& s = g_state[device];
    hipError_t e = hipSetDevice(device);
    if (e != hipSuccess) return hip_fail("hipSetDevice", e);
    if (!s.ready) {
        hipDeviceProp_t prop;
        e = hipGetDeviceProperties(&prop, device);
        if (e != hipSuccess) return hip_fail("hipGetDeviceProperties", e);
        if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0)
            return fail(RPA_ERR_UNSUPPORTED, std::string("device is ") + prop.gcnArchName + ", kernels are gfx950 only");
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail("hipGetSymbolAddress(scratch)", e);
        std::string msg;
        if (rpa::kernels_init(device, msg) != 0) return fail(RPA_ERR_HIP, msg);
        s.ptr = (unsigned char*)p;
        s.num_cus = prop.multiProcessorCount;
        s.blob.reserve(kListBytes);
        s.ready = true;
    }
    *out = &s;
    return RPA_OK;
}

} // namespace

extern "C" const char* rpa_noalloc_last_error(void) { return g_noalloc_err.c_str(); }

extern "C" int rpa_update_and_attend_noalloc(const rpa_shape* shape, int device, void* out, const void* q,
                                             const void* k_new, const void* v_new, void* k_pages, void* v_pages,
                                             const int32_t* page_table, const int32_t* cu_q_lens,
                                             const int32_t* kv_lens, int32_t num_seqs, float sm_scale,
                                             void* stream) {
    using namespace rpa;
    if (!shape) return fail(RPA_ERR_INVALID_ARG, "rpa_update_and_attend_noalloc: null shape");
    std::string msg;
    int rc = check_shape(*shape, msg);
    if (rc != RPA_OK) return fail(rc, msg);
    if (shape->kv_fp8)
        return fail(RPA_ERR_UNSUPPORTED,
                    "rpa_update_and_attend_noalloc: the 8-bit cache needs a staging copy of the new rows, which this "
                    "entry point has no room for; use a context");
    if (num_seqs == 0) return RPA_OK;
    if (!out || !q || !k_new || !v_new || !k_pages || (!v_pages && !shape->kv_merged) || !page_table)
        return fail(RPA_ERR_INVALID_ARG, "rpa_update_and_attend_noalloc: null tensor pointer");
    const uintptr_t align = (uintptr_t)out | (uintptr_t)q | (uintptr_t)k_new | (uintptr_t)v_new |
                            (uintptr_t)k_pages | (uintptr_t)v_pages;
    if (align & 15) return fail(RPA_ERR_INVALID_ARG, "rpa_update_and_attend_noalloc: tensors must be 16-byte aligned");
    if (!std::isfinite(sm_scale) || !(sm_scale > 0.f))
        return fail(RPA_ERR_INVALID_ARG, "rpa_update_and_attend_noalloc: sm_scale must be finite and positive");
    if (num_seqs < 0 || num_seqs > shape->max_seqs)
        return fail(RPA_ERR_BAD_LENGTHS, "rpa_update_and_attend_noalloc: num_seqs outside [0, max_seqs]");
    if (!cu_q_lens || !kv_lens) return fail(RPA_ERR_INVALID_ARG, "rpa_update_and_attend_noalloc: null length array");

    DeviceState* s = nullptr;
    rc = device_state(device, &s);
    if (rc != RPA_OK) return rc;

    // Split partials that fit the array: one (m, l) pair and head_dim floats per row.
    const int64_t row_cap = (int64_t)(kPartialBytes / ((size_t)(shape->head_dim + 2) * sizeof(float)));
    // One stream only.  A large mixed batch runs as one launch that holds both kinds
    // of workgroup, where that kernel is built; else the wide kernel follows the
    // narrow one and the plan is made for that.
    rpa_options opt{};
    Plan& plan = s->plan;
    KernelArgs a{};
    a.kv_merged = shape[0].kv_merged;
    a.head_dim = shape->head_dim;
    a.hg = shape->num_q_heads / shape->num_kv_heads;
    bool one_launch = false;
    for (int pass = 0; pass < 2; ++pass) {
        rc = build_plan(*shape, cu_q_lens, kv_lens, num_seqs, opt, s->num_cus, row_cap, plan, msg);
        if (rc != RPA_OK) return fail(rc, msg);
        a.wide_tq_log2 = __builtin_ctz((unsigned)wide_q_tokens(a.hg, plan.stats.wide_rows));
        one_launch = plan.stats.concurrent && mixed_launch_built(a, plan.stats.narrow_waves);
        if (one_launch || !plan.stats.concurrent) break;
        opt.mixed_overlap = 1;
    }
    const size_t n_narrow = plan.narrow.size(), n_wide = plan.wide.size(), n_items = plan.items.size();
    if (n_narrow + n_wide == 0) return RPA_OK;

    const size_t units_bytes = (n_narrow + n_wide) * sizeof(rpa_work_unit);
    const size_t items_off = (units_bytes + 15) & ~(size_t)15;
    const size_t bins_off = items_off + n_items * sizeof(rpa_combine_item);
    const size_t n_bins = n_narrow ? plan.bins.size() - 1 : 0;
    const size_t total_bytes = (bins_off + plan.bins.size() * sizeof(int32_t) + 3) & ~(size_t)3;
    if (total_bytes > kListBytes) {
        char buf[200];
        snprintf(buf, sizeof buf,
                 "rpa_update_and_attend_noalloc: the work list of this batch takes %zu bytes, the static workspace "
                 "holds %zu; use a context",
                 total_bytes, kListBytes);
        return fail(RPA_ERR_WORKSPACE, buf);
    }
    std::string& blob = s->blob;
    blob.assign(total_bytes, '\0');
    char* h = &blob[0];
    if (n_narrow) std::memcpy(h, plan.narrow.data(), n_narrow * sizeof(rpa_work_unit));
    if (n_wide) std::memcpy(h + n_narrow * sizeof(rpa_work_unit), plan.wide.data(), n_wide * sizeof(rpa_work_unit));
    if (n_items) std::memcpy(h + items_off, plan.items.data(), n_items * sizeof(rpa_combine_item));
    std::memcpy(h + bins_off, plan.bins.data(), plan.bins.size() * sizeof(int32_t));

    hipStream_t st = (hipStream_t)stream;
    unsigned char* const base = s->ptr; // never `scratch` itself: that name is no device address on the host
    (void)hipGetLastError();            // a stale error of an earlier call is not this call's
    const size_t words = total_bytes / 4;
    for (size_t w0 = 0; w0 < words; w0 += kPokeWords) {
        PokePayload p;
        const int n = (int)(words - w0 < (size_t)kPokeWords ? words - w0 : (size_t)kPokeWords);
        std::memcpy(p.w, h + w0 * 4, (size_t)n * 4);
        hipLaunchKernelGGL(rpa_poke_kernel, dim3(1), dim3(256), 0, st, p, (uint32_t*)(base + w0 * 4), n);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail("work list launch", e);
    }

    a.q = (const uint16_t*)q;
    a.k_new = (const uint16_t*)k_new;
    a.v_new = (const uint16_t*)v_new;
    a.k_pages = (uint16_t*)k_pages;
    a.v_pages = (uint16_t*)v_pages;
    a.out = (uint16_t*)out;
    a.page_table = page_table;
    a.part_ml = (float*)(base + kListBytes);
    a.part_o = a.part_ml + (size_t)row_cap * 2;
    a.num_q_heads = shape->num_q_heads;
    a.num_kv_heads = shape->num_kv_heads;
    a.page_size_log2 = __builtin_ctz((unsigned)shape->page_size);
    a.max_pages_per_seq = shape->max_pages_per_seq;
    a.num_pages = shape->num_pages;
    a.scale_log2 = sm_scale * 1.4426950408889634f;
    a.causal = shape->non_causal ? 0 : 1;
    a.kv_fp8 = 0;
    a.out_scale = 1.f;
    a.wide_persist_grid = plan.wide_persistent_pays() ? s->num_cus : 0;
    a.units = (const rpa_work_unit*)base;
    a.bins = (const int32_t*)(base + bins_off);
    int hrc;
    if (one_launch) {
        a.wide_units = (const rpa_work_unit*)base + n_narrow;
        hrc = launch_mixed(a, (int)n_bins, plan.stats.narrow_waves, (int)n_wide, stream, nullptr);
        if (hrc != 0) return hip_fail("mixed kernel launch", (hipError_t)hrc);
    } else {
        hrc = launch_narrow(a, (int)n_bins, plan.stats.narrow_waves, stream, nullptr);
        if (hrc != 0) return hip_fail("narrow kernel launch", (hipError_t)hrc);
        a.units = (const rpa_work_unit*)base + n_narrow;
        hrc = launch_wide(a, (int)n_wide, stream, nullptr);
        if (hrc != 0) return hip_fail("wide kernel launch", (hipError_t)hrc);
    }
    int max_rows = 0;
    for (const rpa_combine_item& it : plan.items) max_rows = max_rows > it.rows ? max_rows : it.rows;
    hrc = launch_combine((const rpa_combine_item*)(base + items_off), (int)n_items, a.part_o, a.part_ml,
                         (uint16_t*)out, a.num_q_heads, a.head_dim, max_rows, stream, nullptr);
    if (hrc != 0) return hip_fail("combine kernel launch", (hipError_t)hrc);
    return RPA_OK;
}
