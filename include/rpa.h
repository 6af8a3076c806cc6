/*
 * rpa.h - C ABI of the MI355X (gfx950) ragged paged attention library.
 *
 * One call updates a paged KV cache with the newly projected K/V of a ragged
 * batch and computes causal grouped-query softmax attention for every query
 * token over its sequence's cached plus new KV (paper Sec. 3, Algorithm 1
 * "RPA Forward Pass with KV Cache Update Fusion").
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses on the context's GPU, "host"
 *     pointers are ordinary host memory.  No pointer is retained after a call
 *     returns, except that device buffers must stay valid until the work
 *     enqueued on `stream` has finished.
 *   - All tensors are dense, row-major, 16-byte aligned; the 16-bit element
 *     type is bfloat16.
 *   - Every function returns RPA_OK (0) or a negative rpa_status.  Nothing
 *     throws or aborts across this boundary.  On an argument, length, shape or
 *     workspace error (every code but RPA_ERR_HIP) nothing is enqueued and no
 *     tensor is touched.  RPA_ERR_HIP means a HIP runtime call failed part way:
 *     kernels of the call launched before the failure stay enqueued, and out
 *     and the cache are then undefined.  rpa_last_error() gives a message.
 *   - The library allocates only its own workspace, in rpa_create(); the call
 *     path performs no allocation, creates no stream and synchronises neither
 *     the device nor the caller's stream.  For a batch that is not small the
 *     host does wait, a few microseconds, for the call's own work list (tens of
 *     KB) to reach the device on a stream of the context
 *     (rpa_options.stream_ordered_upload selects other forms: an event the
 *     caller's stream waits for, or no copy at all), and, when it has run eight
 *     calls ahead of the GPU, for the oldest of them to finish.
 *   - A context serves one stream at a time: calls on one context must be
 *     issued in stream order (the work lists it uploads are reused); a caller
 *     that moves a context between streams orders those streams itself.
 */
#ifndef RPA_H
#define RPA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RPA_OK = 0,
    RPA_ERR_INVALID_ARG = -1, /* null pointer, negative count, unknown enum           */
    RPA_ERR_BAD_LENGTHS = -2, /* cu_q_lens not non-decreasing from 0, kv_len < q_len,
                                 more tokens/sequences/pages than the shape allows     */
    RPA_ERR_UNSUPPORTED = -3, /* shape outside what the kernels are built for          */
    RPA_ERR_HIP = -4,         /* a HIP runtime call failed (message has the detail)    */
    RPA_ERR_WORKSPACE = -5    /* the plan does not fit the workspace sized at create   */
} rpa_status;

/* Static problem shape, fixed at rpa_create().  max_tokens and max_seqs are the
 * paper's static upper bounds s and n (Sec. 3.6 "Recompilation Handling"): a
 * call may use fewer, the padding is neither read nor written.               */
typedef struct {
    int32_t num_q_heads;       /* h_q                                                */
    int32_t num_kv_heads;      /* h_kv; num_q_heads must be a multiple of it        */
    int32_t head_dim;          /* d_k: 64, 128 or 256                                */
    int32_t page_size;         /* tokens per cache page: a power of two >= 16        */
    int32_t max_tokens;        /* s: rows of q / k_new / v_new / out                 */
    int32_t max_seqs;          /* n: rows of page_table                              */
    int32_t max_pages_per_seq; /* row stride of page_table                           */
    int32_t num_pages;         /* pages in each of k_pages and v_pages               */
    int32_t non_causal;        /* 0: causal mask aligned to the end of the sequence
                                  (the default; Alg. 1 "mask S if needed"); 1: no mask,
                                  every query token sees all kv_len positions (the
                                  paper's non-causal prefill measurements, Sec. 4.2)  */
    int32_t kv_fp8;            /* 0: k_pages / v_pages hold bf16.  1: they hold one byte
                                  per element, OCP E4M3 (bias 7, largest value 448, no
                                  infinities), scaled per tensor (Sec. 3.6
                                  "Quantization"): a byte b stands for value(b) * scale.
                                  k_new / v_new stay bf16; a new row x is stored as the
                                  byte nearest (ties to even) to fp32(x) * fp32(1/scale),
                                  saturated to +-448, and attention reads the stored
                                  values for every position, the call's own tokens
                                  included.  At head_dim 128 both kernels have this
                                  variant; at 64 and 256 every batch then runs on the
                                  narrow kernel (built for the bandwidth-bound decode). */
    float k_scale;             /* scale of k_pages (> 0, finite); read if kv_fp8 only   */
    float v_scale;             /* scale of v_pages                                       */
    int32_t kv_merged;         /* 0: separate k_pages and v_pages.  1: the paper's merged
                                  KV layout (Sec. 3.1.3 "KV merge"): k_pages is ONE pool
                                  bf16 [num_pages, page_size, num_kv_heads, 2, head_dim]
                                  in which a token's K and V of a head lie side by side
                                  (index 0 = K, 1 = V); v_pages is ignored and may be
                                  NULL.  bf16 cache at head_dim 128 only, and every batch
                                  then runs on the narrow kernel (the layout is built and
                                  measured for the bandwidth-bound decode case).        */
} rpa_shape;

/* Kernel variants (Sec. 3.4 "Distribution-aware Compilation": decode-only,
 * prefill-only and mixed).  AUTO picks from the batch's length distribution.
 * Forcing a variant changes speed only: every variant is correct on any batch. */
typedef enum {
    RPA_VARIANT_AUTO = 0,
    RPA_VARIANT_DECODE = 1,  /* every query tile through the narrow split-KV kernel   */
    RPA_VARIANT_PREFILL = 2, /* every query tile through the wide MFMA tile kernel    */
    RPA_VARIANT_MIXED = 3    /* sequences of up to 16 / (Hq / Hkv) query tokens (one
                                narrow tile) narrow, the rest wide                    */
} rpa_variant;

/* One unit of work: a query tile of one sequence against a range of that
 * sequence's KV positions.  A wide unit is one workgroup; narrow units are
 * grouped into bins of equal KV volume, one workgroup per bin.  Exposed for
 * rpa_plan_host().                                                            */
typedef struct {
    int32_t seq;        /* sequence index r                                           */
    int32_t q_start;    /* packed token index of the tile's first query token         */
    int32_t q_pos0;     /* index of that token inside its sequence                     */
    int32_t n_q;        /* query tokens in the tile                                   */
    int32_t kv_begin;   /* first KV position of the range (multiple of 16)            */
    int32_t kv_end;     /* one past the last KV position the tile may see in range    */
    int32_t ctx;        /* kv_len - q_len of the sequence: positions >= ctx are new   */
    int32_t seq_q0;     /* cu_q_lens[r]                                               */
    int32_t part_row;   /* first row of this unit's split partial, or -1: write out   */
    int32_t flags;      /* bit 0: this unit writes the tile's new K/V into the pages;
                           bit 1: wide kernel (else narrow); bit 2 (wide units): the
                           tile is its sequence's only one, so its K/V rows are read
                           once in this call and the wide kernel streams them        */
    int32_t bin;        /* narrow units: index of the workgroup that runs the unit     */
    int32_t reserved;
} rpa_work_unit;

/* Merge job for one query tile that was split over KV ranges.                */
typedef struct {
    int32_t part_row;   /* first partial row of split 0                               */
    int32_t n_splits;
    int32_t rows;       /* rows per split = n_q * num_q_heads                         */
    int32_t q_start;    /* packed token index of the tile's first token               */
} rpa_combine_item;

typedef struct {
    int32_t variant;         /* rpa_variant actually used                             */
    int32_t num_narrow_units;
    int32_t num_wide_units;
    int32_t num_combine_items;
    int32_t max_splits;      /* largest number of KV ranges one tile was cut into     */
    int32_t kv_chunk;        /* KV positions per narrow workgroup (bin)               */
    int32_t num_narrow_bins; /* workgroups (x num_kv_heads / narrow_waves) of the narrow kernel */
    int32_t narrow_waves;    /* waves per narrow workgroup                            */
    int64_t partial_rows;    /* fp32 partial rows used                                */
    int64_t workspace_bytes; /* device workspace owned by the context                 */
    int32_t wide_rows;       /* query rows (tokens x heads of a group) per wide tile  */
    int32_t concurrent;      /* 1: narrow and wide kernels were enqueued side by side on
                                two streams; 2: as one launch that holds both kinds of
                                workgroup                                              */
} rpa_plan_stats;

/* Tuning knobs; all-zero = defaults.  They change speed only, never results
 * beyond floating-point summation order.                                      */
typedef struct {
    int32_t variant;   /* rpa_variant; AUTO selects from the length distribution      */
    int32_t kv_chunk;  /* cap on KV positions per narrow unit (rounded up to 16); 0 = none */
    int32_t wide_kv_chunk; /* KV positions per wide unit (rounded up to 64); 0 = auto */
    int32_t narrow_waves;  /* waves (= KV heads) per narrow workgroup: a divisor of
                              num_kv_heads, at most 8 (4 at head_dim 256: every wave
                              keeps head_dim * 128 bytes of LDS); 0 = auto            */
    int32_t units_per_cu;  /* narrow bins per resident workgroup slot (1 = exactly one
                              wave of workgroups); 0 = default                        */
    int32_t ablate;        /* measurement only (ablation by leaving a stage out, as in
                              the paper's kernel analysis, Sec. 4.1 / 4.2 ablation
                              tables).  The switches are compiled into a separate
                              measurement build of the library only; the product
                              library returns RPA_ERR_UNSUPPORTED for any value but
                              0.  Outputs are then meaningless (and the cache is not
                              updated where the write is left out); every access
                              stays in bounds.  Bits:
                                1   narrow kernel: loads and stores only, no math ("w/o FA")
                                2   narrow kernel: no cache write ("w/o KV update")
                                4   narrow kernel: no K/V loads ("w/o DMA")
                                64  wide kernel: no K/V loads (compute runs on stale LDS)
                                128 wide kernel: K/V loads only, no compute
                                256 wide kernel: no output store
                                512 wide kernel: no cache write                        */
    int32_t wide_rows;     /* query rows per wide tile: 256 (eight waves, one workgroup
                              per CU) or 128 (four waves, two workgroups per CU);
                              0 = chosen per call: 256 if that leaves every CU at
                              least four workgroups, or one of long (64 K/V tiles
                              or more on average), full tiles, else 128; 128 beside
                              narrow work (a mixed batch), with the 8-bit
                              cache and at head_dim 64.  head_dim 256 has the 128-row
                              shape only (one workgroup per CU) and rejects 256       */
    int32_t wide_order;    /* launch order of the wide units: 1 = longest tile first
                              overall; 2 = by sequence, heaviest sequence first,
                              longest tile first inside a sequence (the tiles of a
                              sequence then run at about the same time and share its
                              K/V in L2); 0 = 2 where the wide launch is the persistent
                              one (see wide_persistent), the KV heads come in
                              multiples of 8, the sequences are of about one length
                              and nothing narrow runs beside it, else 1               */
    int32_t mixed_overlap; /* a batch with narrow and wide work: 0 = side by side as
                              one launch wherever that kernel is built (below), else
                              with the wide kernel on a stream of the context (forked
                              from and joined to the caller's stream) when both
                              parts are large enough to repay the two extra stream
                              packets; 1 = always one after the other on the caller's
                              stream; 2 = always side by side; 3 = always side by side
                              and as two kernels on two streams.  Side by side means
                              one launch that holds narrow and wide workgroups where
                              that kernel is built (K and V in separate pools,
                              head_dim 64 / 128, with the 8-bit cache 128 only;
                              1, 2 or 4 waves per narrow workgroup; 128-row wide
                              tiles), else the two-stream form                       */
    int32_t stream_ordered_upload; /* how the call's work list reaches the kernels:
                              3 = it is copied to device memory on a stream of the
                              context and the host waits (a few microseconds) for
                              that copy before it enqueues the kernels; 1 = copied,
                              and the host never waits: the caller's stream is made
                              to wait for the copy with an event (one more packet
                              on the stream, about 5 us of GPU idle time per call);
                              2 = not copied: the kernels read it from the pinned
                              host memory it was written to (nothing to wait for;
                              1-3 us more kernel time on a large batch); 0 = 2 for
                              a call estimated to keep the GPU busy for less than
                              30 us, which latency bounds, else 3                   */
    int32_t wide_persistent; /* 256-row wide tiles at head_dim 64 / 128 with a bf16 cache:
                              0 = when the items are short (under 64 K/V tiles each
                              on average) one persistent workgroup per CU walks the
                              (tile, KV head) items (the next item's Q tile and
                              first K/V tiles are requested while the current one
                              finishes), else one workgroup per item;
                              1 = always one workgroup per item                        */
} rpa_options;

typedef struct rpa_ctx rpa_ctx;

/* Create a context on HIP device `device` for `shape`; allocates the workspace
 * (work lists, pinned staging, split partials; with kv_fp8 a staging copy of
 * the new K/V rows) and two streams of default priority.  *out is set on
 * success only.  A context is used by one host thread at a time; calls on one
 * context are ordered by the streams they are given, and the workspace (split
 * partials, staging copy) is shared by them, so calls that may overlap on the
 * GPU (different streams without an ordering between them) need a context each. */
int rpa_create(rpa_ctx** out, const rpa_shape* shape, int device);

/* Free the workspace.  Waits for the device first (kernels of the last calls may
 * still be reading the context's work lists and partials).  NULL is allowed.   */
void rpa_destroy(rpa_ctx* ctx);

/* The hot path (Algorithm 1).  For each sequence r < num_seqs with
 *   l_q = cu_q_lens[r+1] - cu_q_lens[r],  l_kv = kv_lens[r],  ctx = l_kv - l_q:
 *   - token t of the sequence (packed row cu_q_lens[r] + t of k_new / v_new) is
 *     copied bit for bit into slot (ctx + t) % page_size of page
 *     page_table[r][(ctx + t) / page_size] of k_pages / v_pages
 *     (Sec. 3.3 "Update U_kv"; Alg. 1 "update new KV entries");
 *   - out[cu_q_lens[r] + t, h, :] = softmax_j(sm_scale * q[.., h, :] . K_j) V_j over
 *     positions j <= ctx + t of KV head h / (num_q_heads / num_kv_heads), K/V being
 *     the sequence's pages after the update (Alg. 1 inner loop and final
 *     diag(l)^-1 step; Sec. 3.1.2 for the head grouping).
 * Products accumulate in fp32, softmax weights are rounded to bf16 before the
 * second contraction, the result is rounded to bf16 (nearest even).
 * No cache byte other than the sum(l_q) new slots changes.  Rows of out at or
 * beyond cu_q_lens[num_seqs], sequences at or beyond num_seqs, page_table
 * entries at or beyond ceil(l_kv / page_size) and cache slots at or beyond l_kv
 * are never read or written.  A page that is written in this call must belong
 * to one sequence only.  Calling twice with the same arguments gives the same
 * result.  The call only enqueues work on `stream`.
 *
 *   out        dev  bf16 [max_tokens, num_q_heads,  head_dim]   written
 *   q          dev  bf16 [max_tokens, num_q_heads,  head_dim]
 *   k_new      dev  bf16 [max_tokens, num_kv_heads, head_dim]
 *   v_new      dev  bf16 [max_tokens, num_kv_heads, head_dim]
 *   k_pages    dev  bf16 [num_pages, page_size, num_kv_heads, head_dim]  updated in place
 *   v_pages    dev  bf16 [num_pages, page_size, num_kv_heads, head_dim]  updated in place
 *              (with rpa_shape.kv_fp8: one E4M3 byte per element, same index order)
 *   page_table dev  int32 [max_seqs, max_pages_per_seq]; ids outside
 *                   [0, num_pages) are clamped into range (wrong result, no fault)
 *   cu_q_lens  host int32 [num_seqs + 1], cu_q_lens[0] = 0, non-decreasing
 *   kv_lens    host int32 [num_seqs], each includes the sequence's new tokens
 *   num_seqs   0 <= num_seqs <= max_seqs (0: success, nothing enqueued)
 *   sm_scale   softmax scale applied to q . k in fp32; finite and > 0
 *   stream     hipStream_t (NULL = the default stream)
 */
int rpa_update_and_attend(rpa_ctx* ctx, void* out, const void* q, const void* k_new,
                          const void* v_new, void* k_pages, void* v_pages,
                          const int32_t* page_table, const int32_t* cu_q_lens,
                          const int32_t* kv_lens, int32_t num_seqs, float sm_scale,
                          void* stream);

/* The hot call for callers that cannot allocate device memory: code under HIP
 * stream capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and error codes as rpa_update_and_attend, with the shape
 * and the HIP device index in place of a context.  It calls no hipMalloc /
 * hipFree and creates no stream or event: the device work list and the split
 * partials live in one static device array of 8 MiB + 64 KiB that each GPU the
 * library runs on holds until the process ends; the work list reaches it inside
 * kernel arguments.  Limits, beyond which RPA_ERR_WORKSPACE (work list of the
 * batch above 64 KiB, about 1300 units) or RPA_ERR_UNSUPPORTED (kv_fp8, whose
 * staging copy of the new rows has no room here) is returned and nothing is
 * enqueued; split partials that would not fit 8 MiB make the partitioner cut
 * less instead.  The kernels of a mixed batch run one after the other on
 * `stream`.  Every call on a GPU uses that GPU's one array: calls that may
 * overlap on one GPU (different streams without an ordering between them) race;
 * calls in stream order are safe, and nothing in the array has to be cleared
 * between calls (every word read by a call is written by the same call first).
 * rpa_noalloc_last_error() gives the message of this thread's last failure.  */
int rpa_update_and_attend_noalloc(const rpa_shape* shape, int device, void* out, const void* q,
                                  const void* k_new, const void* v_new, void* k_pages, void* v_pages,
                                  const int32_t* page_table, const int32_t* cu_q_lens,
                                  const int32_t* kv_lens, int32_t num_seqs, float sm_scale, void* stream);
const char* rpa_noalloc_last_error(void);

/* Message of the last failed call on this context (never NULL; "" if none).
 * With ctx == NULL: the message of the last failed rpa_create / rpa_plan_host
 * on this thread.                                                             */
const char* rpa_last_error(const rpa_ctx* ctx);

/* Statistics of the last successful rpa_update_and_attend on this context.   */
int rpa_plan_info(const rpa_ctx* ctx, rpa_plan_stats* out);

/* Set the tuning knobs for later calls (tests and tuning); NULL restores the
 * defaults.  The set applies to every batch, whatever its regime, and replaces
 * any per-regime sets.                                                         */
int rpa_set_options(rpa_ctx* ctx, const rpa_options* opt);

/* One set of knobs per regime (Sec. 3.1.4 / 3.4: separate block sizes for
 * decode-only, prefill-only and mixed batches, tuned offline and applied at
 * bring-up).  `regime` is RPA_VARIANT_DECODE, _PREFILL or _MIXED: the regime a
 * batch is classified into from its lengths; `opt` is then used for the batches
 * of that regime (NULL: the defaults); opt->variant must be RPA_VARIANT_AUTO or
 * equal to `regime`.  Regimes never set keep the set of rpa_set_options().
 * python -m paper_2604_15464_amd.tune writes such a table for a shape.          */
int rpa_set_regime_options(rpa_ctx* ctx, int32_t regime, const rpa_options* opt);

/* Kernel timing for benchmarks (not part of the paper's method).  While enabled,
 * every call attaches a start and a stop HIP event to each kernel it launches
 * on the call's stream (at most 1024 calls are kept between two reads).  rpa_profile_read()
 * synchronises on the last recorded event and adds up, over the calls since the
 * previous read, the milliseconds spent in the narrow kernel, the wide kernel
 * and the combine kernel (the one launch of a mixed batch counts as the narrow
 * kernel); *calls receives the number of calls covered.                        */
int rpa_profile_enable(rpa_ctx* ctx, int on);
int rpa_profile_read(rpa_ctx* ctx, float* narrow_ms, float* wide_ms, float* combine_ms,
                     int32_t* calls);

/* Measurement aid (not part of the paper's method): a plain device-to-device
 * copy of `bytes` bytes (a multiple of 16; both pointers 16-byte aligned, the
 * ranges must not overlap) by an ordinary streaming kernel on `stream`.  It is
 * the known-size workload that hardware HBM byte counters and the attention
 * kernels' bandwidth figures are calibrated against.  If ms is not NULL the
 * call waits for the kernel and stores its duration in milliseconds.         */
int rpa_copy_probe(rpa_ctx* ctx, void* dst, const void* src, size_t bytes, void* stream,
                   float* ms);

/* Measurement aid (not part of the paper's method): a kernel of bf16 MFMAs
 * (32x32x16) and nothing else, one workgroup of eight waves per compute unit,
 * `steps` (1 .. 2^20) steps of 32 MFMAs per wave, on `stream`; no memory is read
 * or written.  It shows the matrix rate the machine sustains with every compute
 * unit busy, the figure the wide kernel's TFLOP/s stand against on that machine.
 * *flops (if not NULL) receives the FLOPs of the launch; if ms is not NULL the
 * call waits for the kernel and stores its duration in milliseconds.         */
int rpa_mfma_probe(rpa_ctx* ctx, int32_t steps, void* stream, float* ms, double* flops);

/* Host-only planning, no GPU needed: the work partition that
 * rpa_update_and_attend would use on a device with `num_cus` compute units
 * (Alg. 1's loops over sequences, Q blocks and KV blocks, flattened into units;
 * the split of a tile's KV range over several units is this library's own).
 * Writes at most max_units / max_items records (narrow units first, then wide
 * units, each group in launch order); the counts go to *stats.  opt may be NULL.
 * Returns RPA_ERR_WORKSPACE if a buffer is too small.                         */
int rpa_plan_host(const rpa_shape* shape, const int32_t* cu_q_lens, const int32_t* kv_lens,
                  int32_t num_seqs, const rpa_options* opt, int num_cus, rpa_work_unit* units,
                  int32_t max_units, rpa_combine_item* items, int32_t max_items,
                  rpa_plan_stats* stats);

#ifdef __cplusplus
}
#endif
#endif /* RPA_H */
