// gfx950 kernels of the ragged paged attention hot path (paper Algorithm 1).
//
// Orientation used by every MFMA here (CDNA4, 64-lane waves): the score tile is
// computed transposed, S^T = K Q^T, so that KV positions run along the MFMA's
// M index and query rows along its N index.  In the accumulator layout a lane
// then holds values of ONE query row (column n = lane % 16) for four KV
// positions (4 * (lane / 16) + v), which is exactly the B-operand layout the
// second contraction O^T = V^T P^T needs: the softmax weights never leave the
// registers, and the row statistics (running max m, running sum l of Alg. 1)
// are reduced with two cross-lane steps.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <algorithm>
#include <type_traits>

#include "rpa_internal.h"

namespace rpa {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// Read-only tables are read through the constant address space so that
// wave-uniform reads become scalar loads (and stay so next to the inline asm).
typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
typedef __attribute__((address_space(3))) short4v lds_short4;
typedef const __attribute__((address_space(3))) bf16x8 lds_bf16x8;
typedef __attribute__((ext_vector_type(2))) int int2v;
typedef __attribute__((address_space(3))) int2v lds_int2;

// Measurement switches (the paper's ablation by leaving a stage out, Sec. 4):
// compiled in only with -DRPA_ABLATE, i.e. in the separate library the ablation
// script loads.  In the product library the conditions are compile-time false.
#ifdef RPA_ABLATE
#define RPA_ABLATED(a, bits) (((a).ablate & (bits)) != 0)
#else
#define RPA_ABLATED(a, bits) false
#endif

// Both attention kernels let softmax weights grow to 2^kRescaleGap before they
// move a row's reference maximum and rescale the accumulator.
constexpr float kRescaleGap = 8.0f;

// ---------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------

// 16-byte asynchronous global -> LDS copy: lane i's 16 bytes land at
// lds_byte_off + 16 * i.  Completion is tracked by vmcnt only; the compiler
// does not know about the LDS write, so every consumer waits explicitly with
// wait_vmcnt<N>() before reading the stage.  The LDS address goes through m0,
// which the asm declares as written, so that the compiler never assumes a value
// of its own survives there (it reserves m0 and warns about the clobber; the
// declaration is what keeps its own m0 uses correct).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void async_load16(const void* gptr, uint32_t lds_byte_off) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gptr), "s"(lds_byte_off)
                 : "memory", "m0");
}

// 16-byte store of data that this call will not read again (outputs, cache
// rows): marked non-temporal so that it does not linger as a dirty line in L2
// until the end-of-kernel write-back (plain stores: +8 us per call on 8 x 2048
// prefill, +16 us on one 8 K sequence; write-through stores, sc0 sc1, with or
// without the hint: the same as this).
__device__ __forceinline__ void store16_streaming(void* p, const uint4& v) {
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t x = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(x, (u32x4_t*)p);
}

// The same for data that is read once (the narrow kernel streams every K/V byte
// exactly once): the non-temporal hint keeps the stream from displacing, and
// being handled like, reusable lines in L2.  Measured on the decode workload:
// 417 -> 378 us.  The wide kernel re-reads K/V from L2 and must not use it.
__device__ __forceinline__ void async_load16_stream(const void* gptr, uint32_t lds_byte_off) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt"
                 :
                 : "v"(gptr), "s"(lds_byte_off)
                 : "memory", "m0");
}

// The same with the address split into a wave-uniform 64-bit base (scalar
// registers) and a 32-bit per-lane byte offset: no per-lane address arithmetic.
__device__ __forceinline__ void async_load16_base(const void* sbase, uint32_t voff, uint32_t lds_byte_off) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0"
                 :
                 : "s"(sbase), "v"(voff), "s"(lds_byte_off)
                 : "memory", "m0");
}

// ... and the non-temporal hint of async_load16_stream
__device__ __forceinline__ void async_load16_base_stream(const void* sbase, uint32_t voff, uint32_t lds_byte_off) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0 nt"
                 :
                 : "s"(sbase), "v"(voff), "s"(lds_byte_off)
                 : "memory", "m0");
}

#pragma clang diagnostic pop

// A pointer whose value is the same in every lane, moved to scalar registers in
// case the compiler did not prove that on its own (the "s" operand of the asm
// above must never be handed a vector register).
__device__ __forceinline__ const char* uniform_ptr(const char* p) {
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const char*)(((uint64_t)hi << 32) | lo);
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

__device__ __forceinline__ uint32_t lds_offset(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// two floats -> packed bf16 pair (round to nearest even), low half = a
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    f32x2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// max over the two 32-lane halves of a wave, in every lane, with the register
// swap v_permlane32_swap (no LDS round trip as a cross-half shuffle would take).
// Written as asm: with both operands equal the compiler's model of the builtin
// folds the second result into the first.  The leading s_nop covers the hazard
// of a VALU write directly before the swap.
__device__ __forceinline__ float max_across_halves(float x) {
    float lo = x, hi = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(lo), "+v"(hi));
    return fmaxf(lo, hi);
}

// Eight E4M3 bytes (an 8-bit KV cache row piece) -> eight bf16, exact: every
// E4M3 value, subnormals included, is a bf16 value.  Byte j becomes element j.
__device__ __forceinline__ bf16x8 e4m3x8_to_bf16x8(const uint2& r) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r.x, 1.0f, false);
    const bf16x2 b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r.x, 1.0f, true);
    const bf16x2 c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r.y, 1.0f, false);
    const bf16x2 d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r.y, 1.0f, true);
    return bf16x8{a[0], a[1], b[0], b[1], c[0], c[1], d[0], d[1]};
}

__device__ __forceinline__ bf16x8 e4m3x8_to_bf16x8(int2v r) {
    return e4m3x8_to_bf16x8(make_uint2((uint32_t)r[0], (uint32_t)r[1]));
}

__device__ __forceinline__ int clamp_page(int page, int num_pages) {
    return min(max(page, 0), num_pages - 1);
}

// ---------------------------------------------------------------------------
// Narrow kernel: query tile of up to 16 rows (16 / h_g tokens x the h_g heads of
// one KV head).  One wave per KV head; every wave runs its own LDS ring fed by
// asynchronous 16-byte loads (the GPU analogue of the paper's double-buffered
// B_kv fetch, Sec. 2.3 / Alg. 1 "start DMA ... wait DMA"), so there is no
// workgroup barrier in the loop.  Used for decode (q_len 1) and short query
// runs; bandwidth-bound.  A unit covers KV positions [kv_begin, kv_end) and
// either writes the final rows or an un-normalised partial (m, l, O).
// ---------------------------------------------------------------------------
//
// KV8: the cache (and the staged copy of the new rows) holds one E4M3 byte per
// element (Sec. 3.6 "Quantization").  Rows are half as long, the ring is twice
// as deep, and operands are widened to bf16 after the LDS read; everything else
// is the same code.
//
// MERGED (bf16 cache, head_dim 128): one pool whose token rows hold K and V side
// by side for every KV head, [num_pages, page_size, Hkv, 2, D] (the paper's KV
// merge, Sec. 3.1.3): a token's K and V of one head are 512 contiguous bytes, one
// wave-wide load brings two tokens' K|V pairs, and K and V rows alternate in the
// LDS stage.  a.k_pages is the pool, a.v_pages is not used.
// (The body is a device function so that the mixed-batch kernel below can run it
// in some of its workgroups: `units` is the narrow unit list, `bin` the bin and `g`
// the KV head of the calling wave, both wave-uniform; the waves of a workgroup
// need not share a bin.)
template <int D, int NST, bool KV8, bool MERGED>
__device__ __forceinline__ void narrow_body(const KernelArgs& a, const rpa_work_unit* units, int bin, int g) {
    static_assert(!MERGED || (!KV8 && D == 128), "the merged layout is built for bf16 at head_dim 128");
    constexpr int ROWB = D * (KV8 ? 1 : 2);     // bytes of one token row of one head
    constexpr int NC = ROWB / 16;               // 16-byte chunks per row
    constexpr int NG = D / 8;                   // groups of 8 elements per row
    constexpr int TPI = MERGED ? 64 / (2 * NC) : 64 / NC; // tokens covered by one wave-wide load
    constexpr int NLD = MERGED ? kNarrowKvTile / TPI / 2 : kNarrowKvTile / TPI; // loads per K (or V) tile
    constexpr int TILEB = kNarrowKvTile * ROWB; // bytes of a K (or V) tile
    constexpr int STAGEB = 2 * TILEB;
    constexpr int LOADS_PER_STAGE = 2 * NLD;
    constexpr int PITCH = MERGED ? 2 * ROWB : ROWB;  // bytes between consecutive token rows of K (or V) in a stage
    constexpr int VOFF = MERGED ? ROWB : TILEB;      // V rows of a stage relative to its K rows
    constexpr int HEADB = MERGED ? 2 * ROWB : ROWB;  // bytes of one head's slice of a cache token row
    constexpr int KSTEPS = D / 32;              // MFMA 16x16x32 steps over head_dim
    constexpr int MT = D / 16;                  // 16-dim output tiles
    constexpr int VG = D > 128 ? D / 128 : 1;   // 128-dim groups of a V row (16 chunks each)
    constexpr int JW = MT / VG;                 // output tiles per group

    extern __shared__ uint4 smem[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n = lane & 15;                  // query row of this lane (MFMA column)
    const int quad = lane >> 4;

    const int hg = a.hg;
    const int Hq = a.num_q_heads, Hkv = a.num_kv_heads;
    const int ps_log2 = a.page_size_log2;
    const int ps_mask = (1 << ps_log2) - 1;
    const int num_pages = a.num_pages;
    const char* const k_pages = (const char*)a.k_pages;
    const char* const v_pages = (const char*)a.v_pages;
    const char* const k_new = (const char*)a.k_new;
    const char* const v_new = (const char*)a.v_new;
    const uint32_t tokstride = (uint32_t)Hkv * HEADB; // bytes between consecutive tokens of the cache
    const uint32_t newstride = (uint32_t)Hkv * ROWB;  // ... of k_new / v_new
    const uint64_t k_delta = (uint64_t)k_pages - (uint64_t)k_new;
    const uint64_t v_delta = (uint64_t)v_pages - (uint64_t)v_new;
    const int tok_n = n / hg; // row n = (token n / hg, head g*hg + n % hg)
    const int hh = n - tok_n * hg;
    constexpr int QSTAGEB = KSTEPS * 1024;      // a unit's Q rows, staged per wave
    const uint32_t lds_wave = lds_offset(smem) + wave * (NST * STAGEB + QSTAGEB);
    const char* lds_wave_ptr = (const char*)smem + wave * (NST * STAGEB + QSTAGEB);
    const uint32_t lds_q = lds_wave + NST * STAGEB;
    const char* lds_q_ptr = lds_wave_ptr + NST * STAGEB;

    // per-lane constants of the gather: load i of a tile brings token
    // m = i*TPI + lane/NC; the lane fetches the 16-byte chunk that the XOR
    // swizzle assigns to its LDS slot.
    const int ld_tok = lane / NC;
    const int ld_chunk = lane % NC;
    uint32_t lane_off[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int m = i * TPI + ld_tok;
        lane_off[i] = (uint32_t)g * ROWB + (uint32_t)((ld_chunk ^ (m % NC)) * 16);
    }
    // merged layout: load j of a tile brings tokens 2j and 2j+1; lane l fetches for
    // token 2j + l/32 a chunk of K (l/16 even) or V (odd), placed by the same swizzle
    const int mg_tok = lane >> 5, mg_sub = (lane >> 4) & 1, mg_pos = lane & 15;
    uint32_t mg_chunk[2 * NLD];
#pragma unroll
    for (int j = 0; j < 2 * NLD; ++j) mg_chunk[j] = (uint32_t)((mg_pos ^ ((2 * j + mg_tok) % NC)) * 16);

    // The workgroup walks the units of its bin back to back; the waves never
    // synchronise with each other.  The ring does not drain between units: while
    // the last tiles of a unit are computed, the Q rows and the first tiles of the
    // next unit are already on their way (the Q rows through an LDS staging area of
    // the wave, by the same asynchronous loads, so that every load of the loop is
    // one the explicit vmcnt bookkeeping knows), and the unit's stores go out
    // behind them.
    //
    // Waiting by count: "vmcnt <= N" with N = the loads requested after the wanted
    // one.  Loads return in order, so as long as the wanted load is outstanding all
    // N younger ones are too and the count stays above N; stores requested in
    // between (never counted here) can only make the wait longer, not shorter.
    struct UnitCtx {
        int ctx, kv_begin, kv_end, seq_q0, ntiles;
        const_i32_ptr pt_row;
    };
    auto load_unit = [&](int idx) {
        // through the constant address space: scalar loads, no vmcnt traffic
        const const_i32_ptr p = (const_i32_ptr)(uintptr_t)(units + idx);
        rpa_work_unit r;
        r.seq = p[0], r.q_start = p[1], r.q_pos0 = p[2], r.n_q = p[3], r.kv_begin = p[4], r.kv_end = p[5];
        r.ctx = p[6], r.seq_q0 = p[7], r.part_row = p[8], r.flags = p[9], r.bin = p[10], r.reserved = p[11];
        return r;
    };
    auto unit_ctx = [&](const rpa_work_unit& w) {
        UnitCtx c;
        c.ctx = w.ctx, c.kv_begin = w.kv_begin, c.kv_end = w.kv_end, c.seq_q0 = w.seq_q0;
        c.ntiles = max(0, (w.kv_end - w.kv_begin + kNarrowKvTile - 1) / kNarrowKvTile);
        c.pt_row = (const_i32_ptr)(uintptr_t)(a.page_table + (size_t)w.seq * a.max_pages_per_seq);
        return c;
    };

    // tile t of a unit into ring slot `slot`
    auto issue_tile = [&](const UnitCtx& c, int t, int slot) {
        if (RPA_ABLATED(a, 4)) return; // measurement: no K/V traffic (the math runs on whatever the LDS holds)
        const int pos0 = c.kv_begin + t * kNarrowKvTile;
        const int pidx = __builtin_amdgcn_readfirstlane(pos0 >> ps_log2);
        const int page = clamp_page(c.pt_row[pidx], num_pages); // a tile never straddles pages
        const uint32_t ldsK = lds_wave + slot * STAGEB;
        const uint32_t ldsV = ldsK + VOFF;
        const int last = c.kv_end - 1 - pos0; // tokens past the range re-read its last token
        if constexpr (MERGED) {
            const size_t page_tok = ((size_t)page << ps_log2);
#pragma unroll
            for (int j = 0; j < 2 * NLD; ++j) {
                const int pos = pos0 + min(2 * j + mg_tok, last);
                const bool cached = pos < c.ctx;
                // cached: the token's K|V pair of this head in the pool; new: the K or the V row of the call's inputs
                const uint64_t addr =
                    cached ? (uint64_t)k_pages + (page_tok + (size_t)(pos & ps_mask)) * tokstride + (uint32_t)g * HEADB +
                                 (uint32_t)mg_sub * ROWB + mg_chunk[j]
                           : (uint64_t)(mg_sub ? v_new : k_new) + (uint64_t)(c.seq_q0 + pos - c.ctx) * newstride +
                                 (uint32_t)g * ROWB + mg_chunk[j];
                async_load16_stream((const void*)addr, ldsK + j * 1024);
            }
            return;
        }
        if (pos0 + kNarrowKvTile <= c.ctx) {
            // whole tile is cached content: one scalar base per pool
            const size_t tile_off = (((size_t)page << ps_log2) + (size_t)(pos0 & ps_mask)) * tokstride;
            const char* kb = k_pages + tile_off;
            const char* vb = v_pages + tile_off;
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                const int m = min(i * TPI + ld_tok, last);
                const uint32_t voff = (uint32_t)m * tokstride + lane_off[i];
                async_load16_stream(kb + voff, ldsK + i * 1024);
                async_load16_stream(vb + voff, ldsV + i * 1024);
            }
        } else {
            // tile holds new tokens: those come from k_new / v_new, never from the
            // page slots this call writes
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                const int pos = pos0 + min(i * TPI + ld_tok, last);
                const bool cached = pos < c.ctx;
                const size_t tokidx = cached ? (((size_t)page << ps_log2) + (size_t)(pos & ps_mask))
                                             : (size_t)(c.seq_q0 + pos - c.ctx);
                // select the pool by adding a wave-uniform pointer difference
                // (tokstride == newstride here: the merged layout took its own path above)
                const uint64_t off = (uint64_t)tokidx * tokstride + lane_off[i];
                const uint64_t ka = (uint64_t)k_new + off + (cached ? k_delta : 0);
                const uint64_t va = (uint64_t)v_new + off + (cached ? v_delta : 0);
                async_load16_stream((const void*)ka, ldsK + i * 1024);
                async_load16_stream((const void*)va, ldsV + i * 1024);
            }
        }
    };

    // Q rows of a unit into the wave's staging area: k-step kk of lane i lands at
    // kk * 1024 + 16 * i, where the same lane reads it back.  A padding row fetches
    // the tile's first token (always there) and is zeroed after the read.
    auto issue_q = [&](const rpa_work_unit& w) {
        const char* qrow =
            (const char*)(a.q + ((size_t)(w.q_start + (tok_n < w.n_q ? tok_n : 0)) * Hq + g * hg + hh) * D) + quad * 16;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) async_load16(qrow + kk * 64, lds_q + kk * 1024);
    };
    bf16x8 qreg[KSTEPS];
    auto read_q = [&](const rpa_work_unit& w) {
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            uint4 raw = *(const uint4*)(lds_q_ptr + kk * 1024 + lane * 16);
            if (tok_n >= w.n_q) raw = make_uint4(0, 0, 0, 0);
            qreg[kk] = __builtin_bit_cast(bf16x8, raw);
        }
    };
    // wait until at most `tiles` whole tiles (and the Q rows of the next unit, if
    // they were requested behind the wanted load) are outstanding
    auto wait_behind = [&](int tiles, bool q_behind) {
        const int code = 2 * tiles + (q_behind ? 1 : 0);
        if (code == 0) wait_vmcnt<0>();
        else if (code == 1) wait_vmcnt<KSTEPS>();
        else if (code == 2) wait_vmcnt<LOADS_PER_STAGE>();
        else if (code == 3) wait_vmcnt<LOADS_PER_STAGE + KSTEPS>();
        else if (NST >= 3 && code == 4) wait_vmcnt<(NST >= 3 ? 2 : 0) * LOADS_PER_STAGE>();
        else if (NST >= 3 && code == 5) wait_vmcnt<(NST >= 3 ? 2 : 0) * LOADS_PER_STAGE + KSTEPS>();
        else if (NST >= 4 && code == 6) wait_vmcnt<(NST >= 4 ? 3 : 0) * LOADS_PER_STAGE>();
        else if (NST >= 4 && code == 7) wait_vmcnt<(NST >= 4 ? 3 : 0) * LOADS_PER_STAGE + KSTEPS>();
        else wait_vmcnt<0>();
    };
    static_assert(NST <= 4, "wait_behind covers rings of up to four stages");

    const const_i32_ptr bins = (const_i32_ptr)(uintptr_t)a.bins;
    int ui = bins[bin];
    const int unit_end = bins[bin + 1];
    if (ui >= unit_end) return;

    rpa_work_unit un = load_unit(ui);
    UnitCtx cn = unit_ctx(un);
    int sbase = 0; // ring slot of tile 0 of the unit whose loop runs next
    int pre = 0;   // tiles of that unit already requested
    issue_q(un);
    for (; pre < min(NST - 1, cn.ntiles); ++pre) issue_tile(cn, pre, (sbase + pre) % NST);
    wait_behind(RPA_ABLATED(a, 4) ? 0 : pre, false);
    read_q(un);

    for (;;) {
    const rpa_work_unit u = un;
    const UnitCtx c = cn;
    const bool has_next = ui + 1 < unit_end;
    if (has_next) {
        un = load_unit(ui + 1);
        cn = unit_ctx(un);
    }
    const int lim_next = has_next ? min(NST - 1, cn.ntiles) : 0;
    int pre_next = 0; // tiles of the next unit requested so far
    const int ctx = c.ctx;
    const int kv_begin = c.kv_begin, kv_end = c.kv_end, ntiles = c.ntiles;
    const const_i32_ptr pt_row = c.pt_row;

    const bool row_ok = tok_n < u.n_q;
    // last visible KV position of the row (without the causal mask: no limit but kv_end)
    const int limit_n = row_ok ? (a.causal ? ctx + u.q_pos0 + tok_n : 0x3fffffff) : -1;

    // a predecessor with fewer tiles than the ring is deep has not requested all of
    // this unit's first tiles
    for (; pre < min(NST - 1, ntiles); ++pre) issue_tile(c, pre, (sbase + pre) % NST);

    f32x4 acc[MT];
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY; // running max, log2 domain (score * sm_scale * log2 e)
    float l_run = 0.f;       // this lane's share of the running sum

    for (int t = 0; t < ntiles; ++t) {
        // keep the ring full: tile t + NST - 1 of this unit, or, past its end, the
        // next unit's Q rows and first tiles (the slots they take are those of tiles
        // this loop has already consumed)
        const int j = t + NST - 1;
        if (j < ntiles) {
            issue_tile(c, j, (sbase + j) % NST);
        } else {
            const int kmax = min(j - ntiles + 1, lim_next);
            while (pre_next < kmax) {
                if (pre_next == 0) issue_q(un);
                issue_tile(cn, pre_next, (sbase + ntiles + pre_next) % NST);
                ++pre_next;
            }
        }
        if (!RPA_ABLATED(a, 4)) wait_behind(min(NST - 1, ntiles - 1 - t) + pre_next, pre_next > 0);
        else wait_behind(0, pre_next > 0);

        const char* ldsK = lds_wave_ptr + ((sbase + t) % NST) * STAGEB;
        const char* ldsV = ldsK + VOFF;
        const int pos0 = kv_begin + t * kNarrowKvTile;
        if (RPA_ABLATED(a, 1)) { // measurement: loads and stores only
            acc[0][0] += __uint_as_float(*(const uint32_t*)(ldsK + lane * 4)) + __uint_as_float(*(const uint32_t*)(ldsV + lane * 4));
            continue;
        }

        // ---- S^T = K Q^T (Alg. 1: S <- C_q C_k^T) --------------------------------
        // byte offset in a tile of elements 8*gi .. 8*gi+7 of token row r (the XOR
        // swizzle works on 16-byte chunks: a whole group, or two with 8-bit elements)
        auto group_off = [](int r, int gi) {
            return KV8 ? r * ROWB + (((gi >> 1) ^ (r % NC)) * 16) + (gi & 1) * 8 : r * PITCH + ((gi ^ (r % NC)) * 16);
        };
        auto read_group = [&](const char* tile, int r, int gi) {
            if constexpr (KV8) return e4m3x8_to_bf16x8(*(const uint2*)(tile + group_off(r, gi)));
            else return *(const bf16x8*)(tile + group_off(r, gi));
        };
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            const bf16x8 kop = read_group(ldsK, n, 4 * kk + quad);
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop, qreg[kk], s, 0, 0, 0);
        }

        // ---- mask + online softmax (Alg. 1: m~, P, l~) ------------------------
        float sv[4];
        float mx = -INFINITY;
        const int rel = min(limit_n, kv_end - 1) - pos0 - 4 * quad;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            sv[v] = (v <= rel) ? s[v] : -INFINITY; // position pos0 + 4*quad + v; raw score (sm_scale > 0)
            mx = fmaxf(mx, sv[v]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        // The reference maximum only moves when the row maximum exceeds it by more
        // than kRescaleGap (log2 units): weights may reach 2^gap, which fp32 and bf16
        // hold exactly as well, and the rescale of the accumulator, a multiply per
        // element, becomes rare (skipped under a wave-uniform branch).  The result is
        // unchanged: numerator and l share the reference.
        mx *= a.scale_log2;
        const float m_new = (mx > m_run + kRescaleGap) ? mx : m_run;
        const bool dead = m_new == -INFINITY; // nothing visible yet (or a padding row): state stays (0, 0)
        const float m_use = dead ? 0.f : m_new;
        const float alpha = dead ? 1.f : fast_exp2(m_run - m_use);
        float p[4];
        float psum = 0.f;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            p[v] = fast_exp2(__builtin_fmaf(sv[v], a.scale_log2, -m_use));
            psum += p[v];
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) { // skip when no row's reference moved
#pragma unroll
            for (int j = 0; j < MT; ++j) acc[j] *= alpha;
        }

        union {
            uint32_t w[2];
            short4v v;
        } pop;
        pop.w[0] = pack_bf16(p[0], p[1]);
        pop.w[1] = pack_bf16(p[2], p[3]);

        // ---- O^T += V^T P^T (Alg. 1: C_o <- ... + P C_v) --------------------------
        // lane (m = lane%16, quad) reads 16 bytes (8 dims) of its four tokens and
        // transposes them in registers into eight 4-token operands; a row wider
        // than 128 dims is taken in groups of 16 chunks.
#pragma unroll
        for (int vg = 0; vg < VG; ++vg) {
            uint32_t vr[4][4];
            const int ch = 16 * vg + n % NG;
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                const int tok = 4 * quad + tt;
                const uint4 raw = __builtin_bit_cast(uint4, read_group(ldsV, tok, ch));
                vr[tt][0] = raw.x;
                vr[tt][1] = raw.y;
                vr[tt][2] = raw.z;
                vr[tt][3] = raw.w;
            }
            short4v vop[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
                union {
                    uint32_t w[2];
                    short4v v;
                } o;
                o.w[0] = __builtin_amdgcn_perm(vr[1][j / 2], vr[0][j / 2], sel);
                o.w[1] = __builtin_amdgcn_perm(vr[3][j / 2], vr[2][j / 2], sel);
                vop[j] = o.v;
            }
            if constexpr (D >= 128) {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    acc[8 * vg + j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vop[j], pop.v, acc[8 * vg + j], 0, 0, 0);
            } else {
                const bool upper = n >= NG; // lanes 8..15 serve dims j+4 of their chunk
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    short4v pick;
#pragma unroll
                    for (int e = 0; e < 4; ++e) pick[e] = upper ? vop[j + 4][e] : vop[j][e];
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pick, pop.v, acc[j], 0, 0, 0);
                }
            }
        }
    }

    // ---- the next unit's Q rows: requested behind its first tile at the latest ----
    const float m_fin = m_run, l_fin = l_run; // this unit's state; the registers of Q are free for the next unit's rows
    if (has_next) {
        if (pre_next == 0) issue_q(un); // nothing of the next unit was requested inside the loop
        wait_behind(RPA_ABLATED(a, 4) ? 0 : pre_next, false);
        read_q(un);
    }

    // ---- fused cache update (Alg. 1: "update new KV entries"), once per tile.
    // Readers never take positions >= ctx from the pages (they read k_new / v_new),
    // so this store races with nothing.  When the tile's new rows all lie in the
    // last KV tile of this unit (decode: always) they are still in its ring slot,
    // which nothing overwrites before the next unit's first step, and are copied
    // from there (Sec. 3.3: the update goes out from the on-chip block).
    if ((u.flags & 1) && !RPA_ABLATED(a, 2)) {
        const int cch = lane % NC;
        const int p_first = ctx + u.q_pos0;
        const int last_pos0 = kv_begin + (ntiles - 1) * kNarrowKvTile;
        const bool in_ring = ntiles > 0 && p_first >= last_pos0 && p_first + u.n_q <= kv_end && !RPA_ABLATED(a, 4);
        const char* ldsK = lds_wave_ptr + ((sbase + ntiles - 1 + NST) % NST) * STAGEB;
        const char* ldsV = ldsK + VOFF;
        // at most 16 consecutive positions: one page, or two (page ids by scalar loads)
        const int pi_lo = __builtin_amdgcn_readfirstlane(p_first >> ps_log2);
        const int pi_hi = __builtin_amdgcn_readfirstlane((p_first + u.n_q - 1) >> ps_log2);
        const int page_lo = clamp_page(pt_row[pi_lo], num_pages);
        const int page_hi = clamp_page(pt_row[pi_hi], num_pages);
        auto put_rows = [&](int pos, const uint4& kk, const uint4& vv) {
            const int page = (pos >> ps_log2) == pi_lo ? page_lo : page_hi;
            const size_t dst = (((size_t)page << ps_log2) + (pos & ps_mask)) * tokstride + (size_t)g * HEADB + cch * 16;
            store16_streaming((char*)a.k_pages + dst, kk);
            if constexpr (MERGED) store16_streaming((char*)a.k_pages + dst + ROWB, vv); // V sits beside K in the token's row
            else store16_streaming((char*)a.v_pages + dst, vv);
        };
        // two separate loops: the one that copies from the ring must hold no global
        // load, or the compiler's own vmcnt waits would drain the next unit's tiles
        if (in_ring) {
            for (int t = lane / NC; t < u.n_q; t += 64 / NC) {
                const int r = p_first + t - last_pos0;
                const int off = r * PITCH + ((cch ^ (r % NC)) * 16);
                put_rows(p_first + t, *(const uint4*)(ldsK + off), *(const uint4*)(ldsV + off));
                asm volatile("; rows copied from the ring" ::: "memory"); // keeps this block from being merged with the loop below
            }
        } else {
            for (int t = lane / NC; t < u.n_q; t += 64 / NC) {
                const size_t src = ((size_t)(u.q_start + t) * Hkv + g) * ROWB + cch * 16; // bytes
                put_rows(p_first + t, *(const uint4*)(k_new + src), *(const uint4*)(v_new + src));
            }
        }
    }

    // ---- finalize (Alg. 1: diag(l)^-1 B_o) or store the partial state ------------
    float l_tot = l_fin + __shfl_xor(l_fin, 16);
    l_tot += __shfl_xor(l_tot, 32);
    const int head = g * hg + hh;
    if (!row_ok) {
        // nothing to store for a padding row
    } else if (u.part_row < 0) {
        // accumulator elements acc[JW*vg .. JW*vg + JW-1][v] of a lane are JW consecutive dims
        // (a.out_scale is the V scale of an 8-bit cache, else 1)
        const float inv = l_tot > 0.f ? a.out_scale / l_tot : 0.f;
        uint16_t* orow = a.out + ((size_t)(u.q_start + tok_n) * Hq + head) * D;
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int vg = 0; vg < VG; ++vg) {
                const int mrow = 4 * quad + v;
                const int d0 = 128 * vg + 8 * (mrow % NG) + JW * (mrow / NG);
                uint32_t w[JW / 2];
#pragma unroll
                for (int jj = 0; jj < JW / 2; ++jj)
                    w[jj] = pack_bf16(acc[JW * vg + 2 * jj][v] * inv, acc[JW * vg + 2 * jj + 1][v] * inv);
                if constexpr (JW == 8) *(uint4*)(orow + d0) = make_uint4(w[0], w[1], w[2], w[3]);
                else *(uint2*)(orow + d0) = make_uint2(w[0], w[1]);
            }
    } else {
        const size_t prow = (size_t)u.part_row + (size_t)tok_n * Hq + head;
        float* po = a.part_o + prow * D;
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int vg = 0; vg < VG; ++vg) {
                const int mrow = 4 * quad + v;
                const int d0 = 128 * vg + 8 * (mrow % NG) + JW * (mrow / NG);
                const float os = KV8 ? a.out_scale : 1.f; // partial sums carry the V scale
#pragma unroll
                for (int c4 = 0; c4 < JW / 4; ++c4)
                    *(float4*)(po + d0 + 4 * c4) =
                        make_float4(acc[JW * vg + 4 * c4][v] * os, acc[JW * vg + 4 * c4 + 1][v] * os,
                                    acc[JW * vg + 4 * c4 + 2][v] * os, acc[JW * vg + 4 * c4 + 3][v] * os);
            }
        if (quad == 0) {
            a.part_ml[prow * 2] = m_fin;
            a.part_ml[prow * 2 + 1] = l_tot;
        }
    }
    if (!has_next) break;
    ++ui;
    sbase = (sbase + ntiles) % NST;
    pre = pre_next;
    } // units of the bin
    // stores drain with the end of the wave
}

template <int D, int NST, bool KV8, bool MERGED = false>
__global__ void __launch_bounds__(64 * (D > 128 ? 4 : kMaxWaves)) rpa_narrow_kernel(KernelArgs a) {
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    narrow_body<D, NST, KV8, MERGED>(a, a.units, (int)blockIdx.x, (int)(blockIdx.y * (blockDim.x >> 6)) + wave);
}


// ---------------------------------------------------------------------------
// Wide kernel: query tile of 32 * WAVES rows = (32 * WAVES / h_g) tokens x the h_g
// heads of one KV head (the paper's stacking of a group's heads against one K/V
// operand, Sec. 3.1.2).  Every wave owns 32 rows; 32x32x16 MFMA.  Two shapes are
// built: 8 waves (256 rows, one workgroup per CU, ring of 3 stages) and 4 waves
// (128 rows, two independent workgroups per CU, ring of 2 stages); head_dim 256
// has the 4-wave shape only, one workgroup per CU, each wave alone on its SIMD
// with the whole register file.  K/V tiles of
// 64 positions are staged once per workgroup in LDS by asynchronous 16-byte
// loads (every wave brings its share), one barrier per tile.  Used for prefill
// and chunked prefill; bound by the MFMA, vector and LDS pipes together (every
// wave reads the whole K/V tile from LDS, which loads that pipe as much as the
// MFMAs load theirs).
// ---------------------------------------------------------------------------
//
// KV8 (head_dim 128 only): K/V tiles of E4M3 bytes (Sec. 3.6), see the narrow
// kernel.  Rows are 128 bytes, operands are widened to bf16 after the LDS read
// (the V^T fragment comes from the 8-bit transposing read), the MFMAs and the
// softmax are the same.
//
// PERSIST (the 8-wave bf16 shape): one workgroup per CU walks (unit, KV head)
// items instead of ending after one.  The next item's Q tile arrives through the
// ring slots that fall idle during the last steps of the current item, and its
// first K/V tiles are requested before the current item's output rows are
// stored, so that neither a workgroup launch, nor the Q fetch, nor the drain of
// the output stores stands between two items.
// (Body as a device function, like the narrow kernel's: `units` is the wide unit
// list, `block` and `nblocks` what blockIdx.x and gridDim.x are in a launch of
// its own.)
template <int D, int WAVES, int NST, bool KV8, bool PERSIST>
__device__ __forceinline__ void wide_body(const KernelArgs& a, const rpa_work_unit* units, int block, int nblocks) {
    static_assert(!KV8 || D == 128, "the 8-bit wide kernel is built for head_dim 128");
    static_assert(!PERSIST || (!KV8 && WAVES == 8 && NST == 3 && D <= 128), "shape the persistent loop is built for");
    constexpr int NT = 1; // 32-row groups per wave
    constexpr int ROWB = D * (KV8 ? 1 : 2); // bytes of a K/V row of one head
    constexpr int OROWB = D * 2;            // bytes of a q / out row of one head
    constexpr int NC = ROWB / 16;           // 16-byte chunks per K/V row
    constexpr int ONC = OROWB / 16;
    constexpr int TPI = 64 / NC;   // positions per wave-wide load
    constexpr int KT = kWideKvTile;
    constexpr int TILEB = KT * ROWB;
    constexpr int STAGEB = 2 * TILEB;
    constexpr int WPOS = KT / WAVES; // positions each wave brings per tile
    constexpr int NLD = (WPOS + TPI - 1) / TPI;
    constexpr int KSTEPS = D / 16; // 32x32x16 steps over head_dim
    constexpr int DPL = D / 32;    // output dims per lane per 32-dim MFMA tile set

    extern __shared__ uint4 smem[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int Hkv = a.num_kv_heads;
    const int n32 = lane & 31;
    const int h = lane >> 5;

    // An item is a (unit, KV head) pair, in launch order.  A persistent workgroup
    // takes item blockIdx.x of every round of gridDim.x items, rounds alternating in
    // direction so that the long and the short items of the sorted list even out.
    // With KV heads in multiples of eight the direction turns in groups of eight
    // items (which belong to one unit, so the sums stay even): a workgroup then keeps
    // item % 8 == blockIdx.x % 8 and its XCD sees the same KV heads in every round.
    int round = 0;
    auto item_of_round = [&](int r) {
        const int back =
            ((nblocks | Hkv) & 7) == 0 ? nblocks - 8 - (block & ~7) + (block & 7) : nblocks - 1 - block;
        const int idx = r * nblocks + ((r & 1) ? back : block);
        return (PERSIST && idx < a.num_wide_items) ? idx : -1;
    };
    // unit records are read through the constant address space: scalar loads, so
    // that everything derived from them stays in scalar registers
    auto load_unit = [&](int idx) {
        const const_i32_ptr p = (const_i32_ptr)(uintptr_t)(units + idx);
        rpa_work_unit r;
        r.seq = p[0], r.q_start = p[1], r.q_pos0 = p[2], r.n_q = p[3], r.kv_begin = p[4], r.kv_end = p[5];
        r.ctx = p[6], r.seq_q0 = p[7], r.part_row = p[8], r.flags = p[9], r.bin = p[10], r.reserved = p[11];
        return r;
    };
    int g = block % Hkv;
    rpa_work_unit u = load_unit(block / Hkv);
    const int hg = a.hg;
    const int Hq = a.num_q_heads;
    const int ps_log2 = a.page_size_log2;
    const int ps_mask = (1 << ps_log2) - 1;
    const int num_pages = a.num_pages;
    int ctx = u.ctx;
    const int tq_log2 = a.wide_tq_log2;
    const int tq_mask = (1 << tq_log2) - 1;
    const char* const k_pages = (const char*)a.k_pages;
    const char* const v_pages = (const char*)a.v_pages;
    const char* const k_new = (const char*)a.k_new;
    const char* const v_new = (const char*)a.v_new;
    const_i32_ptr pt_row = (const_i32_ptr)(uintptr_t)(a.page_table + (size_t)u.seq * a.max_pages_per_seq);
    const uint32_t tokstride = (uint32_t)Hkv * ROWB;
    const uint64_t k_delta = (uint64_t)k_pages - (uint64_t)k_new;
    const uint64_t v_delta = (uint64_t)v_pages - (uint64_t)v_new;

    // ---- rows of this lane: rho = 32*(NT*wave + nt) + lane%32 = head_in_group * TQ + token
    int tok[NT], head[NT], limit[NT];
    bool row_ok[NT];
    bf16x8 qreg[NT][KSTEPS];
    // LDS swizzle: 16-byte chunk c of tile row r sits at chunk position c ^ swz(r).
    // swz permutes the bits of r so that both kinds of operand read touch every
    // bank once: a K read (ds_read_b128) takes one chunk from 16 consecutive rows,
    // a transposing V read takes four adjacent chunks from four consecutive rows.
    // LDS banks repeat every 256 bytes, i.e. every row at D = 128 (every half row at
    // D = 256, where the swizzle leaves the chunk's top bit alone) and every second
    // row at D = 64, where the row's parity already separates two rows.
    // With 8-bit elements a row is 128 bytes (8 chunks, two rows per bank period)
    // and operand reads are 8 bytes wide: the row's parity separates two rows, and
    // bits 1..3 of the row index, permuted, spread the eight rows of a K read and
    // the position pairs of a transposing V read over the eight chunk positions.
    auto swz = [](int r) {
        if (KV8) return (((r >> 1) & 1) << 1) | (((r >> 3) & 1) << 2) | ((r >> 2) & 1);
        return D >= 128 ? (((r & 3) << 2) | ((r >> 2) & 3)) : ((((r >> 1) & 1) << 2) | ((r >> 2) & 3));
    };
    int wave_limit = -1;           // positions above it are hidden from every row of the wave
    int wave_min_limit = 1 << 30;  // positions up to it are visible to every live row of the wave
    int kv_begin = 0, kv_end = 0, ntiles = 0;
    // The sequence has this one query tile: its K/V rows are read once in this call
    // (per KV head), like the narrow kernel's, and take the same non-temporal loads
    // (256 sequences of 8 query tokens on 2 K of context: 394 -> 347 us; of 16: 401 ->
    // 384 us).  Tiles that share a sequence re-read its rows from L2 and must not.
    bool stream_kv = false;
    const int ld_tok = lane / NC;
    const int ld_chunk = lane % NC;
    uint32_t lane_voff[NLD]; // byte offset of the lane's chunk of load i from the first token of the wave's share
    // everything that depends on the item (u, g)
    auto setup_item = [&]() __attribute__((always_inline)) {
    ctx = u.ctx;
    pt_row = (const_i32_ptr)(uintptr_t)(a.page_table + (size_t)u.seq * a.max_pages_per_seq);
    wave_limit = -1;
    wave_min_limit = 1 << 30;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int rho = 32 * (NT * wave + nt) + n32;
        const int hh = rho >> tq_log2;
        tok[nt] = rho & tq_mask;
        head[nt] = g * hg + hh;
        row_ok[nt] = tok[nt] < u.n_q;
        limit[nt] = row_ok[nt] ? (a.causal ? ctx + u.q_pos0 + tok[nt] : 0x3fffffff) : -1;
        // the group's 32 rows are 32 consecutive tokens of one head, or whole token
        // ranges of several heads when the tile has fewer than 32 tokens
        const int g_lo = (1 << tq_log2) >= 32 ? ((32 * (NT * wave + nt)) & tq_mask) : 0;
        const int g_hi = (1 << tq_log2) >= 32 ? g_lo + 31 : tq_mask;
        if (g_lo < u.n_q) {
            wave_limit = max(wave_limit, a.causal ? ctx + u.q_pos0 + min(g_hi, u.n_q - 1) : 0x3fffffff);
            wave_min_limit = min(wave_min_limit, a.causal ? ctx + u.q_pos0 + g_lo : 0x3fffffff);
        }
    }
    if (wave_limit < 0) wave_min_limit = -1;
    kv_begin = u.kv_begin;
    kv_end = u.kv_end;
    ntiles = max(0, (kv_end - kv_begin + KT - 1) / KT);
    stream_kv = (u.flags & 4) != 0;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int r = WPOS * wave + i * TPI + ld_tok; // row inside the 64-position tile
        lane_voff[i] = (uint32_t)(i * TPI + ld_tok) * tokstride + (uint32_t)g * ROWB + (uint32_t)((ld_chunk ^ swz(r)) * 16);
    }
    };

    const uint32_t lds_base = lds_offset(smem);

    setup_item();

    // The positions a wave brings for one tile are WPOS <= 16 consecutive ones
    // starting at a multiple of WPOS: they lie in one page (a page holds at least
    // 16 positions), and so do they after clamping to the end of the range.
    static_assert(WPOS <= 16 && 16 % WPOS == 0, "a wave's share of a tile must lie in one page");
    int page_pre = 0; // page id requested at the end of the previous step (see tile_step)
    auto issue_tile = [&](int t, bool have_page) __attribute__((always_inline)) {
        if (RPA_ABLATED(a, 64)) return; // measurement: no K/V traffic
        const int p0w = kv_begin + t * KT + WPOS * wave; // this wave's positions
        const int slot = t % NST;
        const uint32_t ldsK = lds_base + slot * STAGEB + (WPOS * wave) * ROWB;
        const uint32_t ldsV = ldsK + TILEB;
        const int pidx = __builtin_amdgcn_readfirstlane(min(p0w, kv_end - 1) >> ps_log2);
        const int page = clamp_page(have_page ? page_pre : pt_row[pidx], num_pages);
        const bool all_cached = p0w + WPOS <= min(ctx, kv_end);
        const bool all_new = p0w >= ctx && p0w + WPOS <= kv_end;
        if (all_cached || all_new) {
            // the usual case: the whole share comes from one pool and nothing is
            // clamped, so one scalar base per pool serves every load
            const uint64_t tok0 = all_cached ? (((uint64_t)(uint32_t)page << ps_log2) + (uint32_t)(p0w & ps_mask))
                                             : (uint64_t)(uint32_t)(u.seq_q0 + p0w - ctx);
            const uint64_t boff = tok0 * tokstride;
            const char* kb = uniform_ptr((all_cached ? k_pages : k_new) + boff);
            const char* vb = uniform_ptr((all_cached ? v_pages : v_new) + boff);
            if (stream_kv) {
#pragma unroll
                for (int i = 0; i < NLD; ++i) {
                    async_load16_base_stream(kb, lane_voff[i], ldsK + i * 1024);
                    async_load16_base_stream(vb, lane_voff[i], ldsV + i * 1024);
                }
            } else {
#pragma unroll
                for (int i = 0; i < NLD; ++i) {
                    async_load16_base(kb, lane_voff[i], ldsK + i * 1024);
                    async_load16_base(vb, lane_voff[i], ldsV + i * 1024);
                }
            }
        } else {
            // the share straddles the cached/new boundary or the end of the range:
            // per-lane pool and position, positions past the end re-read the last one
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                const int pos = min(p0w + i * TPI + ld_tok, kv_end - 1);
                const bool cached = pos < ctx;
                const size_t tokidx = cached ? (((size_t)page << ps_log2) + (size_t)(pos & ps_mask))
                                             : (size_t)(u.seq_q0 + pos - ctx);
                const uint64_t off =
                    (uint64_t)tokidx * tokstride + (lane_voff[i] - (uint32_t)(i * TPI + ld_tok) * tokstride);
                const uint64_t ka = (uint64_t)k_new + off + (cached ? k_delta : 0);
                const uint64_t va = (uint64_t)v_new + off + (cached ? v_delta : 0);
                async_load16((const void*)ka, ldsK + i * 1024);
                async_load16((const void*)va, ldsV + i * 1024);
            }
        }
    };

    f32x16 o[NT][DPL];
    float m_run[NT], l_run[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m_run[nt] = -INFINITY;
        l_run[nt] = 0.f;
#pragma unroll
        for (int j = 0; j < DPL; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[nt][j][v] = 0.f;
    }

    // LDS read offsets inside a tile, one register per distinct swizzle; the
    // remaining terms of every read are compile-time immediates.
    //   K operand (row 32*mt + n32, chunk 2*kk + h):  koff[kk] + mt * 32 * ROWB
    //   V, dims 32*jb .. 32*jb+31, read rd:           voff[jb][rd] + (32*mt + 16*kh) * ROWB
    // V is read with the transposing LDS load: in each group of 16 lanes, lane
    // 4k + r supplies 8 bytes (4 dims) of one position and lane i receives, as
    // element k, the i-th of the 16 dims that lanes 4k .. 4k+3 supplied.  With
    // lane 4k + r reading position P + k, dims D0 + 4r .. 4r+3, lane i ends up
    // with dim D0 + i of positions P .. P+3: a piece of the V^T operand with no
    // register shuffling.  Read 0 takes positions 4h .. 4h+3 of the 16-position
    // k-step, read 1 positions 8+4h .. 8+4h+3 (the order the weights are in).
    // The swizzle touches the low four bits of the chunk index only, so at
    // D = 256 the offsets of the row's second half are those of the first + 256.
    constexpr int NKO = KSTEPS < 8 ? KSTEPS : 8; // distinct K offsets
    constexpr int NVO = DPL < 4 ? DPL : 4;       // distinct V offset pairs
    uint32_t koff[NKO], voff[NVO][2];
#pragma unroll
    for (int kk = 0; kk < NKO; ++kk) {
        // 8-bit rows: k-step kk is chunk kk, its two 8-element halves go to the wave's two halves
        koff[kk] = KV8 ? lds_base + n32 * ROWB + ((kk ^ swz(n32)) * 16) + 8 * h
                       : (D <= 128 ? lds_base : 0) + n32 * ROWB + (((2 * kk + h) ^ swz(n32)) * 16);
        // opaque from here on: otherwise the compiler splits the sum again and
        // re-adds its parts at every read
        if constexpr (D <= 128) asm volatile("" : "+v"(koff[kk]));
    }
    {
        const int j16 = lane & 15, half16 = (lane >> 4) & 1;
#pragma unroll
        for (int jb = 0; jb < NVO; ++jb)
#pragma unroll
            for (int rd = 0; rd < 2; ++rd) {
                if constexpr (KV8) {
                    // The 8-bit transposing read works on 16 lanes x 8 bytes = 8 rows of
                    // 16 bytes: lanes 2k, 2k+1 supply row k, lane i receives byte i of
                    // rows 0..7.  Row k is made position 8*(k/4) + 4*h + k%4 of the
                    // k-step (the order the weights are in) and the 16 bytes are dims
                    // 32*jb + 16*half16 .. +15: lane i then holds dim 32*jb + 16*half16 + i
                    // for the eight positions of its half of the k-step.  One read per
                    // (k-step, jb): voff[jb][1] is unused.
                    const int k = j16 >> 1;
                    const int r = 8 * (k >> 2) + 4 * h + (k & 3);
                    const int chunk = 2 * jb + half16;
                    voff[jb][rd] = lds_base + r * ROWB + ((chunk ^ swz(r)) * 16) + (j16 & 1) * 8;
                    continue;
                }
                const int r = 4 * h + (j16 >> 2) + 8 * rd; // position modulo 16
                const int chunk = 4 * jb + 2 * half16 + ((j16 & 3) >> 1);
                voff[jb][rd] = (D <= 128 ? lds_base : 0) + r * ROWB + ((chunk ^ swz(r)) * 16) + (j16 & 1) * 8;
                if constexpr (D <= 128) asm volatile("" : "+v"(voff[jb][rd]));
            }
    }

    // K operands are requested in batches of eight k-steps (32 registers).
    constexpr int KB = KSTEPS < 8 ? KSTEPS : 8;
    // At D <= 128 (tile loop unrolled, stage a compile-time constant) an LDS
    // address is one of the registers above, which already include the ring's own
    // address and are opaque to the compiler, plus a compile-time constant that
    // goes into the instruction's offset field: no address arithmetic in the loop.
    // (Formed from the ring's pointer, every operand cost a vector add, a fifth of
    // the loop's vector instructions.)  At D = 256 the stage is a run-time value
    // and the addresses are formed from the pointer as usual.
    constexpr bool IMM = D <= 128;
    const char* lds_ptr = (const char*)smem;
    auto read_k = [&](uint32_t reg, uint32_t rest) __attribute__((always_inline)) {
        if constexpr (KV8) {
            const int2v raw = *(const lds_int2*)(uintptr_t)(reg + rest);
            return e4m3x8_to_bf16x8(raw);
        } else if constexpr (IMM) {
            return (bf16x8) * (lds_bf16x8*)(uintptr_t)(reg + rest);
        } else {
            return *(const bf16x8*)(lds_ptr + rest + reg);
        }
    };
    auto read_v = [&](uint32_t reg, uint32_t rest) __attribute__((always_inline)) {
        if constexpr (IMM) return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(uintptr_t)(reg + rest));
        else return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(lds_ptr + rest + reg));
    };
    auto load_k = [&](bf16x8(&dst)[KB], uint32_t ldsK, int mt, int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int kk = 0; kk < KB; ++kk)
            dst[kk] = read_k(koff[(k0 + kk) % NKO], ldsK + ((k0 + kk) / NKO) * 256 + mt * 32 * ROWB);
    };

    // One 32-position half of a tile: scores, online-softmax update, PV.
    auto compute_half = [&](uint32_t ldsK, uint32_t ldsV, int pos0, int mt_) __attribute__((always_inline)) {
        const int mt = mt_;
        union VOp {
            short4v p[2];
            bf16x8 v;
        };
        VOp vop[2][DPL];
        auto load_v = [&](int kh) {
            const uint32_t src = ldsV + (32 * mt + 16 * kh) * ROWB;
#pragma unroll
            for (int jb = 0; jb < DPL; ++jb) {
                const uint32_t s2 = src + (jb / NVO) * 256;
                if constexpr (KV8) {
                    vop[kh][jb].v = e4m3x8_to_bf16x8(
                        __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_int2*)(uintptr_t)(voff[jb][0] + s2)));
                } else {
                    vop[kh][jb].p[0] = read_v(voff[jb % NVO][0], s2);
                    vop[kh][jb].p[1] = read_v(voff[jb % NVO][1], s2);
                }
            }
        };
        // ---- S^T = K Q^T (Alg. 1: S <- C_q C_k^T) --------------------------------
        f32x16 s[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int v = 0; v < 16; ++v) s[nt][v] = 0.f;
        // the K operands of a batch are requested before its first MFMA, so the LDS
        // latency is paid once per batch, not once per MFMA pair (requesting
        // further ahead, a whole half or across halves, measured slower)
#pragma unroll
        for (int k0 = 0; k0 < KSTEPS; k0 += KB) {
            bf16x8 kop[KB];
            load_k(kop, ldsK, mt, k0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kk = 0; kk < KB; ++kk) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    s[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[kk], qreg[nt][k0 + kk], s[nt], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // The V^T fragments of the half's first 16 positions are requested now and
        // arrive under the softmax; those of the second 16 are requested after it,
        // ahead of the first PV MFMAs.
        load_v(0);
        __builtin_amdgcn_sched_barrier(0);
        // ---- mask + online softmax (Alg. 1: m~, P, l~) ------------------------
        // position of element v is pos0 + 32*mt + 4*h + c with the compile-time
        // c = 8*(v/4) + v%4: visible iff c <= rel.  sm_scale > 0, so the row
        // maximum is taken on the raw scores and scaled once.
        bf16x8 pop[NT][2];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float mx = -INFINITY;
            // Only a half that reaches past some row's diagonal or past the end of
            // the range is masked, under a wave-uniform branch: one copy of the
            // whole half serves both cases, so the accumulators never change
            // registers between a masked and an unmasked variant.
            const int half_last = pos0 + 32 * mt + 31;
            if (half_last > wave_min_limit || half_last >= kv_end) {
                const int rel = min(limit[nt], kv_end - 1) - pos0 - 32 * mt - 4 * h;
#pragma unroll
                for (int v = 0; v < 16; ++v) s[nt][v] = (8 * (v / 4) + (v % 4) <= rel) ? s[nt][v] : -INFINITY;
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[nt][v]);
            mx = max_across_halves(mx) * a.scale_log2;
            // The reference maximum only moves when the row maximum exceeds it by
            // more than kRescaleGap (log2 units): weights may reach 2^gap, which fp32
            // and bf16 hold exactly as well, and the rescale of O becomes rare.  The
            // result is unchanged: numerator and l share the reference.
            const float m_new = (mx > m_run[nt] + kRescaleGap) ? mx : m_run[nt];
            const bool dead = m_new == -INFINITY; // nothing visible yet (or a padding row): state stays (0, 0)
            const float m_use = dead ? 0.f : m_new;
            const float alpha = dead ? 1.f : fast_exp2(m_run[nt] - m_use);
            float psum = 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float pv = fast_exp2(__builtin_fmaf(s[nt][v], a.scale_log2, -m_use));
                s[nt][v] = pv;
                psum += pv;
            }
            l_run[nt] = l_run[nt] * alpha + psum;
            m_run[nt] = m_new;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) { // skip when no row's maximum moved
#pragma unroll
                for (int j = 0; j < DPL; ++j) o[nt][j] *= alpha;
            }
#pragma unroll
            for (int kh = 0; kh < 2; ++kh) {
                union {
                    uint32_t w[4];
                    bf16x8 v;
                } pk;
#pragma unroll
                for (int e = 0; e < 4; ++e) pk.w[e] = pack_bf16(s[nt][8 * kh + 2 * e], s[nt][8 * kh + 2 * e + 1]);
                pop[nt][kh] = pk.v;
            }
        }
        // ---- O^T += V^T P^T (Alg. 1: C_o <- ... + P C_v) --------------------------
        // k-step kh covers positions 32*mt + 8*(2*kh + e/4) + 4*h + e%4, e = 0..7,
        // which is the order of the accumulator elements 8*kh .. 8*kh + 7.
        {
            __builtin_amdgcn_sched_barrier(0);
            load_v(1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                for (int jb = 0; jb < DPL; ++jb)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        o[nt][jb] =
                            __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[kh][jb].v, pop[nt][kh], o[nt][jb], 0, 0, 0);
        }
    };
    // The two halves run through two copies of the code, so that the half's offset
    // is a compile-time constant in every LDS read; the second half is skipped when
    // it lies above the diagonal of every row of the wave.
    auto compute_tile = [&](uint32_t ldsK, uint32_t ldsV, int pos0) __attribute__((always_inline)) {
        compute_half(ldsK, ldsV, pos0, 0);
        if (pos0 + 32 <= wave_limit) compute_half(ldsK, ldsV, pos0, 1);
    };

    // Ring of NST stages: tile t+NST-1 is requested before tile t is consumed, so
    // a tile has NST-1 tile times to arrive.  Each wave waits for its own loads
    // of the next tile, the barrier then makes the whole tile visible.
    constexpr int LPT = 2 * NLD; // loads per wave per tile

    // ---- persistent workgroups: the next item and its Q tile -------------------------
    // The Q tile of the NEXT item travels through the ring as NST-1 more "tiles" of
    // the current item (virtual tiles ntiles .. ntiles+NST-2, in the slots that fall
    // idle once the item's last K/V tiles have been requested): part p holds the
    // rows of the tile's tokens [p * TQH, (p+1) * TQH) for the h_g heads, in the
    // order they lie in memory (a token's h_g head rows are contiguous there, so
    // the loads are whole lines), LPT loads per wave like a K/V tile, which keeps
    // the loop's vmcnt arithmetic unchanged.  Chunk c of a row sits at position
    // c ^ (token % chunks-per-row), so that the operand reads below (32 consecutive
    // tokens, one chunk each) spread over the banks.
    constexpr int QROWS = STAGEB / OROWB;                 // rows of a Q part (one ring slot)
    static_assert(!PERSIST || (ROWB == OROWB && (NST - 1) * QROWS == 32 * WAVES && QROWS % (WAVES * LPT) == 0 &&
                               QROWS / (WAVES * LPT) == 64 / ONC),
                  "a Q tile must fill the ring's idle slots with LPT loads per wave and slot");
    const int hg_log2 = 31 - __builtin_clz((unsigned)hg);
    const int tqh_log2 = tq_log2 - (NST == 3 ? 1 : 0);    // log2 of the tokens per Q part
    int item_n = -1;        // the item after the current one, or -1
    rpa_work_unit un = u;
    int gn = g;
    auto issue_q = [&](const rpa_work_unit& uq, int gq, int part, int slot) __attribute__((always_inline)) {
        const uint32_t lds = lds_base + slot * STAGEB + wave * (LPT * 1024);
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int r_lin = (wave * LPT + i) * (64 / ONC) + lane / ONC;   // row inside the part
            const int tk = (part << tqh_log2) + (r_lin >> hg_log2);
            const int hh = r_lin & (hg - 1);
            const int tkc = min(tk, uq.n_q - 1);                             // rows past the tile re-read its last token
            const int c = (lane % ONC) ^ (tk & (ONC - 1));
            const uint16_t* src = a.q + ((size_t)(uq.q_start + tkc) * Hq + gq * hg + hh) * D + c * 8;
            async_load16(src, lds + i * 1024);
        }
    };
    // Q operands of the current item from the parts that start in ring slot `slot0`.
    auto read_q = [&](int slot0) __attribute__((always_inline)) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int rho = 32 * (NT * wave + nt) + n32;
            const int hh = rho >> tq_log2, tk = rho & tq_mask;
            const int part = tk >> tqh_log2;
            const int r_lin = ((tk - (part << tqh_log2)) << hg_log2) + hh;
            int slot = slot0 + part;
            if (slot >= NST) slot -= NST;
            const char* row = (const char*)smem + slot * STAGEB + r_lin * OROWB;
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) {
                uint4 raw = *(const uint4*)(row + (((2 * kk + h) ^ (tk & (ONC - 1))) * 16));
                if (!row_ok[nt]) raw = make_uint4(0, 0, 0, 0);
                qreg[nt][kk] = __builtin_bit_cast(bf16x8, raw);
            }
        }
    };
    // virtual tile T of the current item: a K/V tile, or a part of the next item's Q tile
    auto issue_virtual = [&](int T, bool have_page) __attribute__((always_inline)) {
        if (T < ntiles) {
            issue_tile(T, have_page);
        } else if (PERSIST && item_n >= 0 && T < ntiles + NST - 1) {
            int slot = T % NST;
            issue_q(un, gn, T - ntiles, slot);
        }
    };
    auto fetch_next_item = [&]() __attribute__((always_inline)) {
        item_n = item_of_round(round + 1);
        if (item_n >= 0) {
            un = load_unit(item_n / Hkv);
            gn = item_n % Hkv;
        }
    };

    if constexpr (PERSIST) {
        // the first item's Q tile, through slots 0 .. NST-2
#pragma unroll
        for (int p0 = 0; p0 < NST - 1; ++p0) issue_q(u, g, p0, p0);
        wait_vmcnt<0>();
        __syncthreads();
        read_q(0);
        __syncthreads(); // every wave holds its operands before the slots take K/V tiles
        fetch_next_item();
    }
#pragma unroll
    for (int s0 = 0; s0 < NST - 1; ++s0) issue_virtual(s0, false);
    if constexpr (!PERSIST) {
        // The Q rows are fetched behind the first tiles so that the two latencies
        // overlap; loads complete in order, hence waiting for Q waits for those tiles.
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const uint16_t* qrow = a.q + ((size_t)(u.q_start + (row_ok[nt] ? tok[nt] : 0)) * Hq + head[nt]) * D;
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) {
                uint4 raw = make_uint4(0, 0, 0, 0);
                if (row_ok[nt]) raw = *(const uint4*)(qrow + kk * 16 + h * 8);
                qreg[nt][kk] = __builtin_bit_cast(bf16x8, raw);
            }
        }
    }
    wait_vmcnt<0>();
    __syncthreads();

    auto tile_step = [&](int t, auto slot) __attribute__((always_inline)) {
        issue_virtual(t + NST - 1, t > 0);
        // relative to the ring: koff / voff carry the ring's own LDS address
        const uint32_t ldsK = (int)slot * STAGEB;
        const uint32_t ldsV = ldsK + TILEB;
        const int pos0 = kv_begin + t * KT;
        // tiles wholly above the wave's diagonal are skipped
        if (pos0 <= wave_limit && !RPA_ABLATED(a, 128)) compute_tile(ldsK, ldsV, pos0);
        // The page id of the share this wave brings in the NEXT step is requested now,
        // after the tile's last operand read and ahead of the waits below, so that its
        // latency passes under them instead of stalling the wave at the start of the
        // next step (a scalar load that is outstanding while operands are read from
        // LDS would turn every wait for those into a full wait: both use one counter).
        {
            const int p_next = min(kv_begin + (t + NST) * KT + WPOS * wave, kv_end - 1);
            // the table row's address is wave-uniform; it is made scalar for the operand below
            // (the halves go through unsigned variables: the builtin returns a signed int)
            const uint64_t pv = (uint64_t)(uintptr_t)pt_row;
            const uint32_t pv_lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)pv);
            const uint32_t pv_hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(pv >> 32));
            const uint64_t ps = ((uint64_t)pv_hi << 32) | pv_lo;
            const uint32_t poff = (uint32_t)__builtin_amdgcn_readfirstlane((p_next >> ps_log2) << 2);
            asm volatile("s_load_dword %0, %1, %2" : "=s"(page_pre) : "s"(ps), "s"(poff));
        }
        // tile t+1 must have landed; virtual tiles t+2 .. may still be in flight
        const int nvt = ntiles + ((PERSIST && item_n >= 0) ? NST - 1 : 0);
        const int behind = min(NST - 2, nvt - 2 - t);
        if (NST >= 4 && behind >= 2) wait_vmcnt<(NST >= 4 ? 2 : 0) * LPT>();
        else if (NST >= 3 && behind == 1) wait_vmcnt<(NST >= 3 ? 1 : 0) * LPT>();
        else wait_vmcnt<0>();
        __syncthreads();
        // The page id has had the barrier's time to return.  It is waited for here, in
        // the step that requested it, also when no step follows: the register it lands
        // in belongs to it only until this statement.
        asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(page_pre));
    };

    // What the second half of an item's epilogue needs once u, g and the row
    // variables describe the next item (all wave-uniform).
    struct Fin {
        int q_start, n_q, part_row, g, flags, q_pos0, ctx;
        const_i32_ptr pt_row;
    };
    // Output rows go through LDS so that the global stores are whole rows, 16 bytes
    // per lane.  Non-persistent: this wave's slice of the (now idle) ring, rows
    // padded by 16 bytes.  Persistent: a region of its own behind the ring (the ring
    // already takes the next item's tiles then), rows unpadded, 16-byte chunk c of
    // row r at position c ^ (r % chunks-per-row).  Either way a wave stages and
    // reads back only its own rows.
    constexpr int SROW = PERSIST ? OROWB : OROWB + 16;
    // First half, for the CURRENT item (u, g, tok, head, row_ok): finalize
    // (Alg. 1: diag(l)^-1 B_o) into the staging rows, or store the partial state.
    // The accumulators are free afterwards.
    auto finalize_stage = [&]() __attribute__((always_inline)) {
        // lane-dependent terms are taken through an opaque copy: in the persistent loop
        // the compiler would otherwise compute every address of this block once, ahead
        // of the item loop, and keep them all in registers across it
        int n32v = n32, hv = h;
        if constexpr (PERSIST) asm volatile("" : "+v"(n32v), "+v"(hv));
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const float l_tot = l_run[nt] + __shfl_xor(l_run[nt], 32);
            if (RPA_ABLATED(a, 256)) continue;
            if (!row_ok[nt] && u.part_row >= 0) continue;
            if (u.part_row < 0) {
                char* stage = (char*)smem + (PERSIST ? NST * STAGEB : 0) + (size_t)(NT * wave + nt) * 32 * SROW;
                const float inv = l_tot > 0.f ? a.out_scale / l_tot : 0.f; // out_scale: V scale of an 8-bit cache, else 1
                // accumulator element v of block jb is dim 32*jb + 8*(v/4) + 4*h + v%4
#pragma unroll
                for (int jb = 0; jb < DPL; ++jb)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        uint2 w;
                        w.x = pack_bf16(o[nt][jb][4 * q4] * inv, o[nt][jb][4 * q4 + 1] * inv);
                        w.y = pack_bf16(o[nt][jb][4 * q4 + 2] * inv, o[nt][jb][4 * q4 + 3] * inv);
                        if constexpr (PERSIST)
                            *(uint2*)(stage + n32v * SROW + (((4 * jb + q4) ^ (n32v & (ONC - 1))) * 16) + 8 * hv) = w;
                        else
                            *(uint2*)(stage + n32v * SROW + (32 * jb + 8 * q4 + 4 * hv) * 2) = w;
                    }
            } else {
                const size_t prow = (size_t)u.part_row + (size_t)tok[nt] * Hq + head[nt];
                float* po = a.part_o + prow * D;
#pragma unroll
                for (int jb = 0; jb < DPL; ++jb)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const float os = KV8 ? a.out_scale : 1.f; // partial sums carry the V scale
                        float4 w = make_float4(o[nt][jb][4 * q4] * os, o[nt][jb][4 * q4 + 1] * os,
                                               o[nt][jb][4 * q4 + 2] * os, o[nt][jb][4 * q4 + 3] * os);
                        *(float4*)(po + 32 * jb + 8 * q4 + 4 * hv) = w;
                    }
                if (hv == 0) {
                    a.part_ml[prow * 2] = m_run[nt];
                    a.part_ml[prow * 2 + 1] = l_tot;
                }
            }
        }
    };
    // Second half: the staged rows go to global memory, whole rows, 16 bytes per lane.
    auto store_rows = [&](const Fin& f) __attribute__((always_inline)) {
        if (f.part_row < 0 && !RPA_ABLATED(a, 256)) {
            constexpr int RPI = 64 / ONC; // rows per wave-wide 16-byte store
            int lv = lane;
            if constexpr (PERSIST) asm volatile("" : "+v"(lv));
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const char* stage = (const char*)smem + (PERSIST ? NST * STAGEB : 0) + (size_t)(NT * wave + nt) * 32 * SROW;
#pragma unroll
                for (int i = 0; i < 32 / RPI; ++i) {
                    const int r = i * RPI + lv / ONC;
                    const int rho = 32 * (NT * wave + nt) + r;
                    const int t_r = rho & tq_mask, h_r = rho >> tq_log2;
                    const int pos = PERSIST ? ((lv % ONC) ^ (r & (ONC - 1))) : (lv % ONC);
                    const uint4 w = *(const uint4*)(stage + r * SROW + pos * 16);
                    if (t_r < f.n_q)
                        store16_streaming(a.out + ((size_t)(f.q_start + t_r) * Hq + f.g * hg + h_r) * D + (lv % ONC) * 8, w);
                }
            }
        }
    };
    // ---- fused cache update for the tile's new tokens (see the narrow kernel)
    auto cache_write = [&](const Fin& f) __attribute__((always_inline)) {
        if ((f.flags & 1) && !RPA_ABLATED(a, 512)) {
            const int c = threadIdx.x % NC;
            for (int t = threadIdx.x / NC; t < f.n_q; t += (64 * WAVES) / NC) {
                const int pos = f.ctx + f.q_pos0 + t;
                const int page = clamp_page(f.pt_row[pos >> ps_log2], num_pages);
                const size_t src = ((size_t)(f.q_start + t) * Hkv + f.g) * ROWB + c * 16; // bytes
                const size_t dst = ((((size_t)page << ps_log2) + (pos & ps_mask)) * Hkv + f.g) * ROWB + c * 16;
                const uint4 kk = *(const uint4*)(k_new + src);
                const uint4 vv = *(const uint4*)(v_new + src);
                store16_streaming((char*)a.k_pages + dst, kk);
                store16_streaming((char*)a.v_pages + dst, vv);
            }
        }
    };

    // The same in two halves for the switch between two items of a persistent
    // workgroup: the rows are read before the next item's first tiles are requested
    // and stored after the wait for those tiles, so that no wait for a cache row has
    // to sit between them.  Two rows per thread at most (tiles of up to 64 tokens).
    constexpr int CWI = 2;
    constexpr int CW_STRIDE = (64 * WAVES) / NC;
    auto cache_rows_load = [&](const Fin& f, uint4 (&kk)[CWI], uint4 (&vv)[CWI], size_t (&dst)[CWI]) __attribute__((always_inline)) {
        const int c = threadIdx.x % NC;
#pragma unroll
        for (int i = 0; i < CWI; ++i) {
            const int t = threadIdx.x / NC + i * CW_STRIDE;
            kk[i] = vv[i] = make_uint4(0, 0, 0, 0);
            dst[i] = 0;
            if ((f.flags & 1) && t < f.n_q && !RPA_ABLATED(a, 512)) {
                const int pos = f.ctx + f.q_pos0 + t;
                const int page = clamp_page(f.pt_row[pos >> ps_log2], num_pages);
                const size_t src = ((size_t)(f.q_start + t) * Hkv + f.g) * ROWB + c * 16;
                dst[i] = ((((size_t)page << ps_log2) + (pos & ps_mask)) * Hkv + f.g) * ROWB + c * 16;
                kk[i] = *(const uint4*)(k_new + src);
                vv[i] = *(const uint4*)(v_new + src);
            }
        }
    };
    auto cache_rows_store = [&](const Fin& f, const uint4 (&kk)[CWI], const uint4 (&vv)[CWI], const size_t (&dst)[CWI]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < CWI; ++i) {
            const int t = threadIdx.x / NC + i * CW_STRIDE;
            if ((f.flags & 1) && t < f.n_q && !RPA_ABLATED(a, 512)) {
                store16_streaming((char*)a.k_pages + dst[i], kk[i]);
                store16_streaming((char*)a.v_pages + dst[i], vv[i]);
            }
        }
    };

    for (;;) {
        if constexpr (D <= 128) {
            // Unrolled over the ring so that a tile's stage is a compile-time constant:
            // the stage base then sits in the offset field of every LDS read instead of
            // costing a vector add per operand (-1.7 %; at D = 256 the doubled loop body
            // costs more than that saves).
            static_assert(NST == 2 || NST == 3, "ring depths the loop is unrolled for");
            for (int t = 0; t < ntiles; t += NST) { // ntiles is the same for every wave: barriers stay matched
                tile_step(t, std::integral_constant<int, 0>{});
                if (t + 1 < ntiles) tile_step(t + 1, std::integral_constant<int, 1>{});
                if constexpr (NST == 3) {
                    if (t + 2 < ntiles) tile_step(t + 2, std::integral_constant<int, 2>{});
                }
            }
        } else {
            for (int t = 0; t < ntiles; ++t) tile_step(t, t % NST);
        }

        Fin f;
        f.q_start = u.q_start, f.n_q = u.n_q, f.part_row = u.part_row, f.g = g, f.flags = u.flags, f.q_pos0 = u.q_pos0;
        f.ctx = ctx, f.pt_row = pt_row;
        finalize_stage(); // the accumulators and the running sums are free from here on
        if (!PERSIST || item_n < 0) {
            store_rows(f);
            cache_write(f);
            break;
        }
        // ---- on to the next item ---------------------------------------------------
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            m_run[nt] = -INFINITY;
            l_run[nt] = 0.f;
#pragma unroll
            for (int j = 0; j < DPL; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[nt][j][v] = 0.f;
        }
        // Its Q parts sit in the slots of the virtual tiles ntiles .. ntiles+NST-2; the
        // last of them may still be in flight.
        const int q_slot0 = ntiles % NST;
        wait_vmcnt<0>();
        __syncthreads();
        u = un;
        g = gn;
        ++round;
        setup_item();
        read_q(q_slot0);
        __syncthreads(); // every wave holds its operands (and is done with the last tile) before the slots are reused
        fetch_next_item();
        // The new item's first tiles are requested BEFORE the old item's rows are
        // stored: loads and stores of a wave complete in the order they were issued, so
        // the wait below, which leaves the youngest stores outstanding, covers these
        // loads without waiting for the stores to drain.
        const bool split_cw = (CWI * CW_STRIDE) >= (1 << tq_log2); // every token of a tile within CWI rows per thread
        uint4 cw_k[CWI], cw_v[CWI];
        size_t cw_dst[CWI];
        if (split_cw) cache_rows_load(f, cw_k, cw_v, cw_dst);
#pragma unroll
        for (int s0 = 0; s0 < NST - 1; ++s0) issue_virtual(s0, false);
        store_rows(f);
        // A full tile that writes its rows issues exactly 32 / (rows per store) row
        // stores per wave after the loads above (each has active lanes); any other
        // case waits for everything.
        if (f.part_row < 0 && f.n_q == (1 << tq_log2) && !RPA_ABLATED(a, 256)) wait_vmcnt<32 / (64 / ONC)>();
        else wait_vmcnt<0>();
        __syncthreads();
        if (split_cw) cache_rows_store(f, cw_k, cw_v, cw_dst);
        else cache_write(f);
    }
}

template <int D, int WAVES, int NST, bool KV8, bool PERSIST = false>
__global__ void __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(D > 128 ? 1 : 2)))
rpa_wide_kernel(KernelArgs a) {
    wide_body<D, WAVES, NST, KV8, PERSIST>(a, a.units, (int)blockIdx.x, (int)gridDim.x);
}

// ---------------------------------------------------------------------------
// Mixed batches (Sec. 3.4, the "mixed" case of the paper's three): one launch
// whose workgroups are narrow ones (four waves) and wide ones of the 128-row
// shape (four waves), so that a CU holds one of each: the narrow part is bound by
// HBM, the wide part by the matrix and vector pipes.  As two kernels on two
// streams the same pairing costs an event from the second stream back to the
// first and the wait for it, 15-20 us of idle GPU per call.  The narrow
// workgroups come first in the grid: the dispatcher spreads consecutive
// workgroups over the CUs before it doubles up, so each CU gets one narrow
// workgroup, which streams for the whole kernel, and the wide ones take the
// second slot of every CU in turn.  (Measured on 128 decode sequences + 4 chunks
// of 512: 404 us; the two kinds alternating in groups of 8, 16 or 32 ids:
// 440-460 us, since some CUs then hold two narrow workgroups; wide first: 455 us;
// wide waves at a raised priority: 418 us; two streams: 418 us.)
// A narrow workgroup is 4 / w tasks of w waves, a task being what a workgroup of
// the narrow kernel's own launch is: one bin and w KV heads, w = 1, 2 or 4 waves
// as the plan chose (the waves never synchronise with each other, so tasks can
// share a workgroup).  A wide item's KV head is item % Hkv, so with Hkv a
// multiple of 8 all items of a head still meet in one XCD's L2, whatever the
// offset.
// ---------------------------------------------------------------------------
template <int D, bool KV8>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) rpa_mixed_kernel(KernelArgs a) {
    const int nn = a.mixed_narrow_wgs;
    if ((int)blockIdx.x < nn) {
        const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
        const int w = a.mixed_narrow_waves;
        const int task = (int)blockIdx.x * (4 / w) + wave / w;
        const int bins = a.mixed_narrow_bins;
        if (task >= bins * (a.num_kv_heads / w)) return; // the last workgroup may be partly empty
        narrow_body<D, KV8 ? 2 * kNarrowStages : kNarrowStages, KV8, false>(a, a.units, task % bins,
                                                                            (task / bins) * w + wave % w);
    } else {
        wide_body<D, 4, kWideStagesHalf, KV8, false>(a, a.wide_units, (int)blockIdx.x - nn, a.mixed_wide_wgs);
    }
}

// ---------------------------------------------------------------------------
// Combine: merge the partial states of a tile that was cut into KV ranges.
// States with different running maxima are rescaled to the common maximum and
// added, as in the rescaling step of Alg. 1.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) rpa_combine_kernel(const rpa_combine_item* __restrict__ items,
                                                          const float* __restrict__ part_o,
                                                          const float* __restrict__ part_ml,
                                                          uint16_t* __restrict__ out, int Hq, int D) {
    // one thread = four consecutive dims of one row; blockIdx.y walks row blocks
    const rpa_combine_item it = items[blockIdx.x];
    const int lanes_per_row = D / 4;
    const int rows_per_block = blockDim.x / lanes_per_row;
    const int dim = (threadIdx.x % lanes_per_row) * 4;
    for (int row = blockIdx.y * rows_per_block + threadIdx.x / lanes_per_row; row < it.rows;
         row += rows_per_block * gridDim.y) {
        const size_t first = (size_t)it.part_row + row;
        float m_run = -INFINITY, den = 0.f;
        float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
        // online merge: the loads of different splits are independent
#pragma unroll 4
        for (int s = 0; s < it.n_splits; ++s) {
            const size_t prow = first + (size_t)s * it.rows;
            const float2 ml = *(const float2*)(part_ml + prow * 2);
            const float4 o = *(const float4*)(part_o + prow * D + dim);
            const float m_new = fmaxf(m_run, ml.x);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float a_old = fast_exp2(m_run - m_use);
            const float a_new = fast_exp2(ml.x - m_use);
            num.x = num.x * a_old + o.x * a_new;
            num.y = num.y * a_old + o.y * a_new;
            num.z = num.z * a_old + o.z * a_new;
            num.w = num.w * a_old + o.w * a_new;
            den = den * a_old + ml.y * a_new;
            m_run = m_new;
        }
        const float inv = den > 0.f ? 1.f / den : 0.f;
        uint2 w;
        w.x = pack_bf16(num.x * inv, num.y * inv);
        w.y = pack_bf16(num.z * inv, num.w * inv);
        *(uint2*)(out + ((size_t)it.q_start * Hq + row) * D + dim) = w;
    }
}

// ---------------------------------------------------------------------------
// 8-bit cache: the new K/V rows are quantised once per call into a staging copy
// (Sec. 3.6: one scale per tensor).  Byte = nearest E4M3 value (ties to even) of
// fp32(x) * inv_scale, saturated to +-448; the attention kernel then reads the
// new rows from the staging copy exactly like cached ones, and the cache write
// is a byte copy.  One thread = eight elements of K and of V.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint2 quantize8(const uint4& raw, float inv_scale) {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
    float f[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(w[i] << 16);          // bf16 -> fp32, exact
        f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float y = f[i] * inv_scale;
        f[i] = (y != y) ? y : fminf(fmaxf(y, -448.f), 448.f); // the conversion itself does not saturate
    }
    int lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], 0, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], lo, true);
    int hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[4], f[5], 0, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[6], f[7], hi, true);
    return make_uint2((uint32_t)lo, (uint32_t)hi);
}

__global__ __launch_bounds__(256) void rpa_quantize_kernel(const uint4* __restrict__ k_new, const uint4* __restrict__ v_new,
                                                           uint2* __restrict__ k8, uint2* __restrict__ v8, size_t n8,
                                                           float inv_k, float inv_v) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += stride) {
        k8[i] = quantize8(k_new[i], inv_k);
        v8[i] = quantize8(v_new[i], inv_v);
    }
}

// ---------------------------------------------------------------------------
// Plain streaming copy, 16 bytes per lane per step.  Not part of the method: it
// is the known-size workload against which HBM byte counters and the narrow
// kernel's bandwidth are calibrated.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rpa_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src,
                                                       size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// ---------------------------------------------------------------------------
// A loop of bf16 MFMAs and nothing else: eight waves per workgroup (two per SIMD,
// as in the wide kernel), 32 MFMAs 32x32x16 per step over four accumulators and
// four register sets per operand, no memory access.  Not part of the method: it
// measures the matrix rate the chip sustains with every CU busy and operands that
// look like data, which is what the wide kernel's TFLOP/s figure stands against
// on a given machine.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(512) void rpa_mfma_kernel(int steps) {
    // operands: pseudo-random bf16 values of either sign in [0.5, 2), different in
    // every lane and register (with near-constant operands the same loop runs at
    // the nominal rate: what the chip sustains depends on how many bits toggle)
    bf16x8 x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            uint32_t h = (threadIdx.x * 32u + i * 4u + k + 1u) * 2654435761u;
            h ^= h >> 15;
            h *= 2246822519u;
            h ^= h >> 13;
            w[k] = (h & 0x80ff80ffu) | 0x3f003f00u;
        }
        x[i] = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
    }
    f32x16 o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[i][e] = 0.f;
    for (int t = 0; t < steps; ++t) {
#pragma unroll
        for (int i = 0; i < 32; ++i)
            o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[i & 3], x[4 + ((i >> 2) & 3)], o[i & 3], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) asm volatile("" ::"v"(o[i])); // the results are wanted by nobody else
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
template <int D>
static size_t narrow_lds_bytes(int waves) {
    return (size_t)waves * narrow_lds_per_wave(D);
}

template <int D>
static size_t wide_lds_bytes(int stages) {
    return (size_t)stages * 2 * kWideKvTile * D * 2;
}

// persistent 8-wave shape: the ring plus a staging region for the output rows
template <int D>
static size_t wide_lds_bytes_persistent() {
    return wide_lds_bytes<D>(kWideStages) + (size_t)8 * 32 * D * 2;
}

// 8-bit K/V rows: the ring is half the size and the output staging of the
// epilogue (32 padded bf16 rows per wave) is what sizes the allocation.
static size_t wide_lds_bytes_kv8(int stages, int waves) {
    return std::max((size_t)stages * 2 * kWideKvTile * 128, (size_t)waves * 32 * (128 * 2 + 16));
}

int kernels_init(int device, std::string& err) {
    (void)device;
    hipError_t e;
    e = hipFuncSetAttribute((const void*)rpa_narrow_kernel<128, kNarrowStages, false>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)narrow_lds_bytes<128>(kMaxWaves));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_narrow_kernel<128, kNarrowStages, false, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)narrow_lds_bytes<128>(kMaxWaves));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_narrow_kernel<64, kNarrowStages, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)narrow_lds_bytes<64>(kMaxWaves));
    // 8-bit cache: rows half as long, ring twice as deep, the same bytes per wave
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_narrow_kernel<128, 2 * kNarrowStages, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)narrow_lds_bytes<128>(kMaxWaves));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_narrow_kernel<64, 2 * kNarrowStages, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)narrow_lds_bytes<64>(kMaxWaves));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_narrow_kernel<256, 2 * kNarrowStages, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)narrow_lds_bytes<256>(kLdsBytesPerCu / narrow_lds_per_wave(256)));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_wide_kernel<128, 8, kWideStages, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)wide_lds_bytes<128>(kWideStages));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_wide_kernel<128, 8, kWideStages, false, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)wide_lds_bytes_persistent<128>());
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_wide_kernel<64, 8, kWideStages, false, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)wide_lds_bytes_persistent<64>());
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_wide_kernel<64, 8, kWideStages, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)wide_lds_bytes<64>(kWideStages));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_wide_kernel<128, 4, kWideStagesHalf, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)wide_lds_bytes<128>(kWideStagesHalf));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_wide_kernel<64, 4, kWideStagesHalf, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)wide_lds_bytes<64>(kWideStagesHalf));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_wide_kernel<128, 8, kWideStages, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)wide_lds_bytes_kv8(kWideStages, 8));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_wide_kernel<128, 4, kWideStagesHalf, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)wide_lds_bytes_kv8(kWideStagesHalf, 4));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_narrow_kernel<256, kNarrowStages, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)narrow_lds_bytes<256>(kLdsBytesPerCu / narrow_lds_per_wave(256)));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_wide_kernel<256, 4, kWideStagesHalf, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)wide_lds_bytes<256>(kWideStagesHalf));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_mixed_kernel<128, false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)std::max(narrow_lds_bytes<128>(4), wide_lds_bytes<128>(kWideStagesHalf)));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_mixed_kernel<64, false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)std::max(narrow_lds_bytes<64>(4), wide_lds_bytes<64>(kWideStagesHalf)));
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)rpa_mixed_kernel<128, true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)std::max(narrow_lds_bytes<128>(4), wide_lds_bytes_kv8(kWideStagesHalf, 4)));
    if (e != hipSuccess) {
        err = std::string("hipFuncSetAttribute: ") + hipGetErrorString(e);
        return (int)e;
    }
    return 0;
}

#define RPA_LAUNCH(kernel, grid, block, lds, st, ev, ...)                                              \
    hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)(lds), st, (ev) ? (hipEvent_t)(ev)[0] : nullptr, \
                          (ev) ? (hipEvent_t)(ev)[1] : nullptr, 0, __VA_ARGS__)

int launch_narrow(const KernelArgs& a, int num_bins, int waves, void* stream, void** ev) {
    if (num_bins <= 0) return 0;
    dim3 grid(num_bins, a.num_kv_heads / waves);
    dim3 block(64 * waves);
    hipStream_t st = (hipStream_t)stream;
    if (a.kv_fp8) {
        if (a.head_dim == 256)
            RPA_LAUNCH((rpa_narrow_kernel<256, 2 * kNarrowStages, true>), grid, block, narrow_lds_bytes<256>(waves), st,
                       ev, a);
        else if (a.head_dim == 128)
            RPA_LAUNCH((rpa_narrow_kernel<128, 2 * kNarrowStages, true>), grid, block, narrow_lds_bytes<128>(waves), st,
                       ev, a);
        else
            RPA_LAUNCH((rpa_narrow_kernel<64, 2 * kNarrowStages, true>), grid, block, narrow_lds_bytes<64>(waves), st,
                       ev, a);
    } else if (a.kv_merged)
        RPA_LAUNCH((rpa_narrow_kernel<128, kNarrowStages, false, true>), grid, block, narrow_lds_bytes<128>(waves), st, ev, a);
    else if (a.head_dim == 256)
        RPA_LAUNCH((rpa_narrow_kernel<256, kNarrowStages, false>), grid, block, narrow_lds_bytes<256>(waves), st, ev, a);
    else if (a.head_dim == 128)
        RPA_LAUNCH((rpa_narrow_kernel<128, kNarrowStages, false>), grid, block, narrow_lds_bytes<128>(waves), st, ev, a);
    else
        RPA_LAUNCH((rpa_narrow_kernel<64, kNarrowStages, false>), grid, block, narrow_lds_bytes<64>(waves), st, ev, a);
    return (int)hipGetLastError();
}

int launch_quantize(const void* k_new, const void* v_new, void* k8, void* v8, size_t elems, float inv_k, float inv_v,
                    int num_cus, void* stream) {
    const size_t n8 = elems / 8;
    if (n8 == 0) return 0;
    const size_t want = (n8 + 255) / 256;
    const size_t cap = (size_t)num_cus * 8;
    dim3 grid((unsigned)(want < cap ? want : cap));
    RPA_LAUNCH(rpa_quantize_kernel, grid, dim3(256), 0, (hipStream_t)stream, (void**)nullptr, (const uint4*)k_new,
               (const uint4*)v_new, (uint2*)k8, (uint2*)v8, n8, inv_k, inv_v);
    return (int)hipGetLastError();
}

int launch_copy(void* dst, const void* src, size_t n16, int num_cus, void* stream, void** ev) {
    if (n16 == 0) return 0;
    const size_t want = (n16 + 255) / 256;
    const size_t cap = (size_t)num_cus * 8;
    dim3 grid((unsigned)(want < cap ? want : cap));
    RPA_LAUNCH(rpa_copy_kernel, grid, dim3(256), 0, (hipStream_t)stream, ev, (uint4*)dst, (const uint4*)src, n16);
    return (int)hipGetLastError();
}

int launch_mfma(int steps, int num_cus, void* stream, void** ev) {
    if (steps <= 0 || num_cus <= 0) return 0;
    RPA_LAUNCH(rpa_mfma_kernel, dim3((unsigned)num_cus), dim3(512), 0, (hipStream_t)stream, ev, steps);
    return (int)hipGetLastError();
}

int launch_wide(const KernelArgs& a_in, int num_units, void* stream, void** ev) {
    if (num_units <= 0) return 0;
    KernelArgs a = a_in;
    a.num_wide_items = num_units * a.num_kv_heads;
    dim3 grid((unsigned)num_units * a.num_kv_heads);
    hipStream_t st = (hipStream_t)stream;
    // One 32-row group per wave: with two, an operand read would feed two MFMAs,
    // but the 512-register shape that needs is beyond what the compiler allocates
    // without spilling.
    const bool half = (a.hg << a.wide_tq_log2) == 128; // 128-row tiles: four waves, two workgroups per CU
    if (a.kv_fp8) {
        if (a.head_dim != 128) return (int)hipErrorInvalidValue; // other sizes run on the narrow kernel
        if (half)
            RPA_LAUNCH((rpa_wide_kernel<128, 4, kWideStagesHalf, true>), grid, dim3(256),
                       wide_lds_bytes_kv8(kWideStagesHalf, 4), st, ev, a);
        else
            RPA_LAUNCH((rpa_wide_kernel<128, 8, kWideStages, true>), grid, dim3(512), wide_lds_bytes_kv8(kWideStages, 8),
                       st, ev, a);
    } else if (a.head_dim == 256) {
        // one shape only: 128 rows, four waves with the whole register file each, and
        // a ring of two 64 KB stages (one workgroup per CU)
        if (!half) return (int)hipErrorInvalidValue;
        RPA_LAUNCH((rpa_wide_kernel<256, 4, kWideStagesHalf, false>), grid, dim3(256), wide_lds_bytes<256>(kWideStagesHalf),
                   st, ev, a);
    } else if (!half && a.wide_persist_grid > 0) {
        // persistent: one workgroup per CU walks the (unit, KV head) items
        dim3 pgrid((unsigned)std::min<int64_t>((int64_t)a.num_wide_items, (int64_t)a.wide_persist_grid));
        if (a.head_dim == 128)
            RPA_LAUNCH((rpa_wide_kernel<128, 8, kWideStages, false, true>), pgrid, dim3(512),
                       wide_lds_bytes_persistent<128>(), st, ev, a);
        else
            RPA_LAUNCH((rpa_wide_kernel<64, 8, kWideStages, false, true>), pgrid, dim3(512),
                       wide_lds_bytes_persistent<64>(), st, ev, a);
    } else if (a.head_dim == 128) {
        if (half)
            RPA_LAUNCH((rpa_wide_kernel<128, 4, kWideStagesHalf, false>), grid, dim3(256),
                       wide_lds_bytes<128>(kWideStagesHalf), st, ev, a);
        else
            RPA_LAUNCH((rpa_wide_kernel<128, 8, kWideStages, false>), grid, dim3(512), wide_lds_bytes<128>(kWideStages), st,
                       ev, a);
    } else {
        if (half)
            RPA_LAUNCH((rpa_wide_kernel<64, 4, kWideStagesHalf, false>), grid, dim3(256),
                       wide_lds_bytes<64>(kWideStagesHalf), st, ev, a);
        else
            RPA_LAUNCH((rpa_wide_kernel<64, 8, kWideStages, false>), grid, dim3(512), wide_lds_bytes<64>(kWideStages), st,
                       ev, a);
    }
    return (int)hipGetLastError();
}

// Narrow and wide workgroups in one launch: a.units / a.bins are the narrow list,
// a.wide_units the wide one.  Built for the bf16 cache (separate pools) at head_dim
// 64 and 128, four waves per narrow workgroup and 128-row wide tiles.
bool mixed_launch_built(const KernelArgs& a, int narrow_waves) {
    const bool half = (a.hg << a.wide_tq_log2) == 128;
    const bool waves_ok = narrow_waves == 1 || narrow_waves == 2 || narrow_waves == 4;
    if (a.kv_merged || !half || !waves_ok) return false;
    return a.kv_fp8 ? a.head_dim == 128 : a.head_dim <= 128;
}

int launch_mixed(const KernelArgs& a_in, int num_bins, int narrow_waves, int num_wide_units, void* stream, void** ev) {
    KernelArgs a = a_in;
    if (!mixed_launch_built(a, narrow_waves) || a.num_kv_heads % narrow_waves != 0 || num_bins <= 0 ||
        num_wide_units <= 0)
        return (int)hipErrorInvalidValue;
    const int tasks = num_bins * (a.num_kv_heads / narrow_waves), per_wg = 4 / narrow_waves;
    a.mixed_narrow_bins = num_bins;
    a.mixed_narrow_waves = narrow_waves;
    a.mixed_narrow_wgs = (tasks + per_wg - 1) / per_wg;
    a.mixed_wide_wgs = num_wide_units * a.num_kv_heads;
    a.num_wide_items = a.mixed_wide_wgs;
    const dim3 grid((unsigned)(a.mixed_narrow_wgs + a.mixed_wide_wgs));
    hipStream_t st = (hipStream_t)stream;
    if (a.kv_fp8)
        RPA_LAUNCH((rpa_mixed_kernel<128, true>), grid, dim3(256),
                   std::max(narrow_lds_bytes<128>(4), wide_lds_bytes_kv8(kWideStagesHalf, 4)), st, ev, a);
    else if (a.head_dim == 128)
        RPA_LAUNCH((rpa_mixed_kernel<128, false>), grid, dim3(256),
                   std::max(narrow_lds_bytes<128>(4), wide_lds_bytes<128>(kWideStagesHalf)), st, ev, a);
    else
        RPA_LAUNCH((rpa_mixed_kernel<64, false>), grid, dim3(256),
                   std::max(narrow_lds_bytes<64>(4), wide_lds_bytes<64>(kWideStagesHalf)), st, ev, a);
    return (int)hipGetLastError();
}

int launch_combine(const rpa_combine_item* items, int num_items, const float* part_o, const float* part_ml,
                   uint16_t* out, int num_q_heads, int head_dim, int max_rows, void* stream, void** ev) {
    if (num_items <= 0) return 0;
    // enough row blocks that the largest item is covered in one pass: the merge is
    // a chain of dependent loads per row, so it wants threads, not iterations
    const int rows_per_block = 256 / (head_dim / 4);
    const int ny = std::min(512, std::max(1, (max_rows + rows_per_block - 1) / rows_per_block));
    dim3 grid(num_items, ny);
    RPA_LAUNCH(rpa_combine_kernel, grid, dim3(256), 0, (hipStream_t)stream, ev, items, part_o, part_ml, out,
               num_q_heads, head_dim);
    return (int)hipGetLastError();
}

} // namespace rpa
