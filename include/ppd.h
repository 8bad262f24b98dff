/*
 * ppd.h -- C ABI of libppd: the decode-node hot path of PPD serving on one MI355X (gfx950).
 *
 * One engine step on a decode node that also runs append-prefill locally (paper section 4.1, "Full
 * Prefill vs. Append Prefill"; section 2.1 for decode): every sequence i of the batch has L_i tokens of
 * KV already cached on the node and n_i new tokens.  n_i = 1 is a decode step, n_i > 1 with L_i > 0 is
 * an append-prefill, L_i = 0 is a full prefill.  (The paper writes n for the cached and m for the new
 * tokens; this interface writes L and n.)  New row j of a sequence attends to keys 0 .. L_i + j: the
 * whole cached prefix plus the new tokens up to and including itself.
 *
 * The step is two calls: ppd_kv_append writes the new tokens' K/V into the page pool, then
 * ppd_mixed_attention computes all rows of all sequences in one launch, reading every key -- cached or
 * new -- from the pool.
 *
 * Conventions
 *  - All tensor pointers are DEVICE pointers unless a parameter says HOST.  They are borrowed: the
 *    library neither frees them nor keeps them after the enqueued work has run.
 *  - q, out, k, v and every page pool must start on a 16-byte boundary (the kernels move 16 bytes per lane);
 *    slot_mapping on an 8-byte, page_tables on a 4-byte boundary.  Anything else is PPD_ERR_RANGE.
 *  - bf16 = the upper 16 bits of an IEEE binary32.  Arithmetic: bf16 inputs, fp32 accumulation and
 *    softmax, probabilities rounded to bf16 before the PV product, bf16 output (round to nearest even).
 *  - Both calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL = the default stream);
 *    the caller synchronises.  Host-side argument checks are complete before anything is enqueued: a
 *    negative return value means no device side effect.
 *  - Values that live in device memory (page ids, slots) cannot be checked on the host; the kernels
 *    never dereference an out-of-range id (the token or key is skipped) and raise a sticky flag that
 *    ppd_device_error_flags reads back.
 *  - ppd_kv_append enqueues one kernel launch.  ppd_mixed_attention plans on the host and uploads the plan when L, n
 *    or the options differ from the previous call on the context (pinned staging buffer, one asynchronous copy);
 *    otherwise -- the other layers of the same engine step -- it enqueues kernel launches only.  Such a step can be
 *    captured into a HIP graph and replayed (the kernels reset their own queue cursors; no memset nodes); with the
 *    option "timing" set, events are recorded as well, so leave it off under capture.
 *  - One context serves one stream at a time.  Calls on a context are not thread-safe.
 *  - Debugging aids, read from the environment by ppd_create: PPD_LOG=1 prints one line per call on stderr (batch
 *    size, tiles of each kind, split sizes, grid, whether the plan was reused); PPD_DEBUG_SLOTS=1 makes every append
 *    look for duplicate slots within the call (two more small launches and a bitmap of one bit per pool slot) and
 *    raises device error flag bit 2 when it finds one.
 *
 * Page pool layout (bf16 elements; P = 16 tokens per page; D = head_dim; Hkv = KV heads):
 *    page stride          S = 2 * Hkv * P * D
 *    K(page, h, tok, d)   at  page*S +            h*P*D + (d/8)*(P*8)  + tok*8 + d%8
 *    V(page, h, tok, d)   at  page*S + Hkv*P*D +  h*P*D + (tok/8)*(D*8) + d*8   + tok%8
 *  A (page, head) block of K or V is P*D*2 bytes contiguous (4 KiB at D = 128); K keeps 8 consecutive d of
 *  a token in one 16-byte granule with the 16 tokens of a page adjacent, V keeps 8 consecutive tokens of
 *  one d in a granule: the two operand shapes the matrix cores consume without a transpose.
 *  With ppd_set_kv_format(PPD_KV_FP8_E4M3) the same offsets address one-byte elements (FP8 codes): blocks and
 *  granules are half as many bytes.
 */
#ifndef PPD_H
#define PPD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ppd_ctx ppd_ctx; /* opaque; owns only its workspace and plan buffers */

typedef enum {
    PPD_OK = 0,
    PPD_ERR_NULL = -1,      /* a required pointer is NULL */
    PPD_ERR_SHAPE = -2,     /* unsupported head_dim / page_size / head counts */
    PPD_ERR_RANGE = -3,     /* n_i < 1, L_i < 0, negative or non-finite scale, sizes out of range, misaligned pointer */
    PPD_ERR_PAGETABLE = -4, /* max_pages < ceil((L_i + n_i) / P) for some sequence */
    PPD_ERR_WORKSPACE = -5, /* workspace allocation failed */
    PPD_ERR_HIP = -6        /* a HIP runtime call failed (see ppd_last_error) */
} ppd_status;

/* Supported: head_dim in {64, 128}; page_size == 16; num_q_heads = G * num_kv_heads with 1 <= G <= 8;
 * num_pages >= 1. */
typedef struct {
    int32_t num_q_heads;
    int32_t num_kv_heads;
    int32_t head_dim;
    int32_t page_size;
    int64_t num_pages;
} ppd_shape;

/* Work-list entry of the one-launch scheduler (host readable through ppd_plan_build). */
typedef struct {
    int32_t kind;     /* 0: narrow tile (rows*G <= 16 columns, HBM-bound: decode), 1: MFMA row-block tile */
    int32_t seq;      /* sequence index */
    int32_t kvh;      /* KV head */
    int32_t row0;     /* first new-token row of the block, within the sequence */
    int32_t nrows;    /* rows in the block */
    int32_t grow0;    /* row0 as an index into q / out */
    int32_t L;        /* cached length of the sequence */
    int32_t kv_total; /* L + n of the sequence */
    int32_t kv_begin; /* key range [kv_begin, kv_end) this tile covers; kv_begin is a multiple of 64 */
    int32_t kv_end;
    int32_t group;    /* merge group, or -1 when the tile covers the whole key range and writes `out` */
    int32_t queue;    /* work queue: 0..7 = MFMA tiles preferred by the workgroups of XCD `queue`, 8 = narrow tiles run by a
                         whole workgroup, 9 = short narrow tiles run one per wave, eight to a claim */
    int64_t part_off; /* float offset of this tile's partial (o, m, l) in the workspace, or -1 */
} ppd_work_item;

typedef struct {
    int64_t n_items;        /* tiles in the work list */
    int64_t n_narrow;       /* of which narrow (decode-like) */
    int64_t n_mfma;         /* of which MFMA row-block tiles */
    int64_t n_groups;       /* merge groups (row blocks whose key range was split) */
    int64_t partial_floats; /* workspace floats for split partials */
    int64_t kv_bytes;       /* sum over sequences of (L_i + n_i) * 2 * Hkv * D * 2: KV read at least once */
    int64_t kv_bytes_tiles; /* KV bytes summed over tiles (row blocks re-read their key range) */
    double flops;           /* 4 * Hq * D * sum_i n_i * (L_i + (n_i + 1) / 2) */
    int32_t narrow_chunk;   /* split size (tokens) chosen for narrow tiles */
    int32_t mfma_chunk;     /* split size (tokens) chosen for MFMA tiles */
    int32_t grid;           /* workgroups launched */
    int32_t plan_host_us;   /* host time spent building and staging this plan, microseconds (0 for ppd_plan_build) */
} ppd_plan_stats;

/* Creates a context bound to HIP device `device` for pools of the given shape. */
ppd_status ppd_create(const ppd_shape *shape, int32_t device, ppd_ctx **out);
ppd_status ppd_destroy(ppd_ctx *ctx);

/* Message of the last failing call on this context (context-owned string; "" if none).  ctx may be NULL
 * to read the message of a failed ppd_create. */
const char *ppd_last_error(const ppd_ctx *ctx);

/* Tuning knobs (all optional).  key: "narrow_chunk", "mfma_chunk" (tokens, multiple of 64, 0 = automatic),
 * "grid" (workgroups, 0 = automatic), "force_kind" (-1 automatic, 1 = route every sequence through the
 * MFMA row-block path; used to test that n = 1 append-prefill equals decode), "pref_mode" (0..3: which
 * kind of tile a workgroup takes first -- 0 MFMA tiles for all, 1 alternating per group of 8 workgroups,
 * 2 split by physical compute unit (default), 3 narrow tiles for all), "narrow_cus" (pref_mode 2: how many of
 * the 32 compute units of an XCD take narrow tiles first; -1 = sized by the planner's cost model so that both
 * kinds finish together), "wave_tiles" (-1 = narrow tiles of at most 384 keys run one per wave, eight to a claim, when the launch has at
 * least six such tiles per workgroup; 0 = never; 1 = whenever there is such a tile), "launch_mode" (0 = one kernel runs both kinds of tiles on separate compute units,
 * 1 = a step that holds both kinds runs as two kernels resident side by side on every compute unit -- row-block
 * tiles on the caller's stream, narrow tiles on a stream of the context's own, joined before the call's work ends
 * -- 2 = the two specialised kernels also for steps of one kind), "narrow_kernel" (1, the default = with launch_mode 0 a step
 * without row-block tiles, i.e. a decode-only step, runs a kernel of its own that hands the first tiles out by
 * workgroup index instead of by atomic claims; same tiles, bit-identical results; 0 = always the one kernel), "timing" (1 = record HIP
 * events on the call's stream right before and after the attention kernel(s), see ppd_last_kernel_ms). */
ppd_status ppd_set_option(ppd_ctx *ctx, const char *key, int64_t value);

/* Element format of the page pools a context works on.  PPD_KV_BF16 (the default) is the paper's setting: KV in
 * 16-bit precision.  PPD_KV_FP8_E4M3 is an extension beyond the paper for the HBM-bound decode rows: the same two
 * layouts with ONE-BYTE elements (every offset above counts elements; a page is Hkv*P*D*2 bytes, 32 KiB at 8 KV
 * heads and D = 128) holding OCP FP8 E4M3 codes -- 1 sign, 4 exponent bits of bias 7, 3 mantissa bits, no
 * infinities, S.1111.111 = NaN, largest finite magnitude 448 -- with one scale per tensor:
 *   ppd_kv_append / ppd_kv_land store   code = e4m3(x * (1 / scale)), the reciprocal and the product in binary32,
 *       rounded to the nearest code, ties to the even code, magnitudes from 448 on saturating to 448, NaN -> NaN code;
 *   ppd_mixed_attention(_static) reads  K = value(code) * k_scale, V = value(code) * v_scale (every code's value is a
 *       bf16 number, so the matrix cores see exact operands; k_scale multiplies the scores, v_scale the output).
 * k, v, q and out stay bf16.  k_scale, v_scale: finite and > 0 (ignored for PPD_KV_BF16).  Takes effect from the next
 * call on; pools written in one format must be read in the same.  Option "launch_mode" must be 0 with FP8 pages. */
#define PPD_KV_BF16 0
#define PPD_KV_FP8_E4M3 1
ppd_status ppd_set_kv_format(ppd_ctx *ctx, int32_t format, float k_scale, float v_scale);

/* Paged KV append (the KV-cache write of the step; paper sections 2.1 and 4.1: prefill populates the
 * cache, decode-side KV stays resident and grows with the context).
 *   k, v          device bf16 [T][Hkv][D], token-major, contiguous
 *   kv_pages      device pool in the layout above, caller-owned
 *   slot_mapping  device int64 [T]; slot = page*P + offset; a negative slot skips the token; a slot beyond
 *                 the pool is skipped and raises device error flag bit 0; duplicate slots in one call are
 *                 a caller error (which copy wins is unspecified)
 * Pure 16-bit copies: the pool afterwards is bit-identical to the definition (FP8 pages: the codes are, see
 * ppd_set_kv_format).  T = 0 is a no-op. */
ppd_status ppd_kv_append(ppd_ctx *ctx, const void *k, const void *v, void *kv_pages,
                         const int64_t *slot_mapping, int64_t T, void *stream);

/* KV landing: the turn-1 side of a decode node.  The KV of a whole request, computed on a prefill node, arrives
 * for all layers at once and is scattered into each layer's page pool (paper section 4.2: KV is transferred on
 * turn 1 only; appendix "Bandwidth Simulation" for the sizes: 128 KiB per token over 32 layers).  Same semantics
 * as num_layers calls of ppd_kv_append in one launch:
 *   k, v                device bf16 [num_layers][T][Hkv][D], contiguous
 *   kv_pages            device: pool of layer 0; pool of layer l starts layer_stride_elems * l elements later
 *                       (layer_stride_elems >= elements of one pool)
 *   slot_mapping        device int64 [T], shared by all layers (a request uses the same pages in every layer) */
ppd_status ppd_kv_land(ppd_ctx *ctx, const void *k, const void *v, void *kv_pages, int64_t layer_stride_elems,
                       int32_t num_layers, const int64_t *slot_mapping, int64_t T, void *stream);

/* Extra delay that emulates a slower interconnect for a KV transfer (paper appendix "Bandwidth Simulation",
 * its equation for the injected delay): max(0, n_tokens * kv_bytes_per_token / beta_target - t_fast), seconds.
 * Host arithmetic only; returns -1 for invalid arguments. */
double ppd_transfer_delay_s(int64_t n_tokens, int64_t kv_bytes_per_token, double beta_target_bytes_per_s,
                            double t_fast_s);

/* Mixed-batch paged attention (paper section 4.1 for append-prefill and full prefill, section 2.1 for
 * decode; the co-batching of the two is the interference experiment of section 4.1).
 *   q, out        device bf16 [T][Hq][D], T = sum n_i, rows grouped by sequence in batch order
 *   kv_pages      device pool; the n_i new tokens of every sequence must already be appended at
 *                 positions L_i .. L_i + n_i - 1
 *   page_tables   device int32 [B][max_pages]; entry p of row i is the page of tokens p*P .. p*P+P-1;
 *                 entries at or beyond ceil((L_i+n_i)/P) are never read; an id outside the pool is clamped
 *                 and raises device error flag bit 1
 *   L, n          HOST int32 [B]
 *   scale         softmax scale (>= 0, finite), applied to q.k before the softmax
 * Result per row is the softmax-weighted average of the visible V rows; run-to-run bitwise deterministic
 * for fixed arguments and options.  B = 0 is a no-op.  A batch whose work list would exceed 2^22 tiles (far beyond
 * any step that fits the chip: a 128K-token full prefill needs ~10^5) is refused with PPD_ERR_RANGE. */
ppd_status ppd_mixed_attention(ppd_ctx *ctx, const void *q, const void *kv_pages, const int32_t *page_tables,
                               int32_t max_pages, const int32_t *L, const int32_t *n, int32_t B, float scale,
                               void *out, void *stream);

/* The same operation for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Arguments, result and error behaviour are those of ppd_mixed_attention; the call itself
 * allocates nothing (no hipMalloc / hipFree / hipHostMalloc, no event creation): the queue counters, the uploaded plan
 * and the split partials live in a fixed device array inside the library, PPD_STATIC_SCRATCH_BYTES per GPU, which
 * every GPU the library runs on holds until the process ends; the pinned staging buffer of the upload belongs to the
 * context and is allocated by ppd_create.  Limits: the plan (56 bytes per tile plus the merge tables) must fit
 * 2 MiB - 4 KiB and the split partials PPD_STATIC_SCRATCH_BYTES - 2 MiB; a batch beyond either is refused with
 * PPD_ERR_WORKSPACE before anything is enqueued.  All contexts of the process share the array of their GPU and it
 * keeps the previous call's contents: the call clears the counters it needs at zero itself, and two calls that
 * overlap in time on one GPU (different streams or threads) race -- serialise them.  Option "timing" does not
 * cover this entry point. */
#define PPD_STATIC_SCRATCH_BYTES (32u << 20)
ppd_status ppd_mixed_attention_static(ppd_ctx *ctx, const void *q, const void *kv_pages, const int32_t *page_tables,
                                      int32_t max_pages, const int32_t *L, const int32_t *n, int32_t B, float scale,
                                      void *out, void *stream);

/* Statistics of the plan built by the last ppd_mixed_attention call on this context. */
ppd_status ppd_get_plan_stats(const ppd_ctx *ctx, ppd_plan_stats *stats);

/* Host-only planner (no device needed): classifies the sequences and emits the tile list the kernel
 * would run, in launch order.  items may be NULL to query the count; at most `capacity` entries are
 * written and stats->n_items holds the full count.  narrow_chunk / mfma_chunk / grid: 0 = automatic;
 * force_kind as in ppd_set_option; num_cus = compute units to balance for (256 on MI355X). */
ppd_status ppd_plan_build(const ppd_shape *shape, const int32_t *L, const int32_t *n, int32_t B,
                          int32_t narrow_chunk, int32_t mfma_chunk, int32_t grid, int32_t force_kind,
                          int32_t num_cus, ppd_work_item *items, int64_t capacity, ppd_plan_stats *stats);

/* Synchronises `stream`, then returns and clears the sticky device error flags (bit 0: append slot out of
 * range, bit 1: page id out of range, bit 2: duplicate slot within an append -- looked for only under
 * PPD_DEBUG_SLOTS=1) in *flags. */
ppd_status ppd_device_error_flags(ppd_ctx *ctx, void *stream, uint32_t *flags);

/* With option "timing" set: waits for the mixed-attention kernel of the last ppd_mixed_attention call and
 * returns its duration in milliseconds (HIP events on the stream it was launched on; the plan upload and
 * the merge kernel are outside the bracket). */
ppd_status ppd_last_kernel_ms(ppd_ctx *ctx, float *ms);

/* With option "timing" set: waits for the mixed-attention kernels of all ppd_mixed_attention calls made since the
 * option was set or since the last call of this function (at most 4096 are kept; later ones are not timed),
 * returns the sum of their durations in *total_ms and their number in *launches, and starts a new series.
 * This is how a benchmark gets the kernel's mean duration over exactly its timed region. */
ppd_status ppd_timed_kernels_ms(ppd_ctx *ctx, double *total_ms, int32_t *launches);

/* ---- PPD routing decision (host only; paper section 3 score equation, section 5 algorithm "PPD Dynamic
 * Routing", appendix "Decision-Engine Discretization") ----
 * Grid: 3 context classes (accumulated context <= 512, <= 4096, larger) x 9 workload types (input/output token
 * ratio classes, given by their centre ratios) x 10 QPS levels (0.5, 1, 2, 4, 6, 8, 10, 12, 16, 20).
 * Cell index = (context_class * 9 + ratio_class) * 10 + qps_level. */
#define PPD_ROUTE_CTX_CLASSES 3
#define PPD_ROUTE_RATIO_CLASSES 9
#define PPD_ROUTE_QPS_LEVELS 10
#define PPD_ROUTE_CELLS (PPD_ROUTE_CTX_CLASSES * PPD_ROUTE_RATIO_CLASSES * PPD_ROUTE_QPS_LEVELS)

/* S = w_ttft * delta_ttft - w_tpot * delta_tpot: delta_ttft is the relative TTFT improvement, delta_tpot the
 * relative TPOT degradation of processing the turn locally on the decode node instead of through a prefill node. */
double ppd_route_score(double w_ttft, double w_tpot, double delta_ttft, double delta_tpot);

/* Offline phase: x_table[cell] = 1 if S > 0 else 0, from measured delta_ttft / delta_tpot per cell
 * (HOST double [PPD_ROUTE_CELLS] each; x_table HOST uint8 [PPD_ROUTE_CELLS]).  Weights must be >= 0. */
ppd_status ppd_route_table_build(const double *delta_ttft, const double *delta_tpot, double w_ttft, double w_tpot,
                                 uint8_t *x_table);

/* Nearest grid cell of a request (n_in new input tokens, n_out expected output tokens, n_ctx accumulated context,
 * current system QPS); the ratio class is the nearest of ratio_centers (HOST double [9], all > 0) on a
 * logarithmic scale.  Returns the cell index or -1 for invalid arguments. */
int32_t ppd_route_cell(const double *ratio_centers, int64_t n_in, int64_t n_out, int64_t n_ctx, double qps);

/* Online phase: turn 1 always returns 0 (prefill-node path: no cached KV yet); later turns return the table
 * entry of the request's nearest cell (1 = run the append-prefill on the decode node).  -1 for invalid arguments. */
int32_t ppd_route_decide(const uint8_t *x_table, const double *ratio_centers, int32_t turn, int64_t n_in,
                         int64_t n_out, int64_t n_ctx, double qps);

/* The online phase for `count` requests in one call (a router's inner loop): x_out[i] = ppd_route_decide(... [i]).
 * All arrays HOST, `count` entries; x_out int8 (-1 marks an invalid request). */
ppd_status ppd_route_decide_batch(const uint8_t *x_table, const double *ratio_centers, int64_t count,
                                  const int32_t *turn, const int64_t *n_in, const int64_t *n_out, const int64_t *n_ctx,
                                  const double *qps, int8_t *x_out);

/* Library version, "major.minor". */
const char *ppd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PPD_H */
