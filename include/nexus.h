/*
 * nexus.h -- C ABI of the MI355X-native hot path of intra-GPU prefill/decode
 * disaggregation: one mixed-batch transformer step in which a chunked-prefill
 * sub-batch and a decode sub-batch run concurrently on disjoint compute-unit
 * (CU) partitions of one GPU (paper Sec. 4 overview and Fig. 6: the inputs of
 * a partitioned step are the CU shares R_p / R_d, the prefill chunk tokens
 * P_T with the KV they attend to, and the decode batch B_d with its KV).
 *
 * Conventions
 *   - Every function returns 0 (NEXUS_OK) or a negative nexus_status; no C++
 *     exception crosses this boundary.  nexus_last_error() returns a
 *     thread-local, library-owned, NUL-terminated description of the last
 *     failure on the calling thread.
 *   - "device" pointers are HIP device memory on the context's GPU, owned by
 *     the caller (e.g. torch tensors); "host" pointers are ordinary memory.
 *     The library owns the context, its streams, its workspace and its packed
 *     copies of the weights.
 *   - bf16 = IEEE bfloat16, 2 bytes, round-to-nearest-even.  All lengths,
 *     offsets and page ids are int32.
 *   - All argument checks happen on the host before anything is launched; a
 *     call that fails launches nothing.  The contents of device-side integer
 *     arrays (lengths, page ids) cannot be checked without a device-to-host
 *     copy; kernels skip page ids outside [0, n_pages) instead of
 *     dereferencing them.  nexus_set_debug_checks() turns on a mode that
 *     makes that copy and validates the arrays before every step.
 *   - Step calls enqueue work and return; nexus_sync() (or a timing request)
 *     waits.  Calls on one context must not overlap from several threads.
 */
#ifndef NEXUS_H
#define NEXUS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    NEXUS_OK = 0,
    NEXUS_EINVAL = -1, /* bad argument (null pointer, negative size, bad enum)       */
    NEXUS_ESHAPE = -2, /* shape outside what the kernels or the context limits allow */
    NEXUS_ENOMEM = -3, /* device or host allocation failed                           */
    NEXUS_EHIP = -4,   /* a HIP runtime call failed; see nexus_last_error()          */
    NEXUS_ESTATE = -5  /* call order violated (e.g. layer weights not loaded)        */
} nexus_status;

typedef struct nexus_ctx nexus_ctx; /* opaque */

/*
 * Decoder-layer shape (Sec. 2.2, Eq. 1-3, in the RMSNorm / rotary / grouped-
 * query / SwiGLU form of the models of Sec. 6.1).  Requirements: head_dim is
 * 64 or 128; n_q_heads is a multiple of n_kv_heads with a ratio of at most 16;
 * hidden and ffn are multiples of 32; page_size is 16.
 */
typedef struct {
    int32_t hidden, n_q_heads, n_kv_heads, head_dim, ffn, n_layers, page_size;
    float rms_eps, rope_theta;
} nexus_model_desc;
/*
 * Precision inside the library: the layer input x, the output y, the rotated queries and the KV cache are bf16;
 * the operands of the four projection GEMMs (normalised activations, attention output, SwiGLU activation and
 * the packed weights) are IEEE half, which the matrix unit runs at the bf16 rate with 8x smaller operand
 * rounding (half holds every bf16 weight of magnitude >= 2^-14 exactly); accumulators, softmax and norm
 * statistics and the residual stream between attention and feed-forward are fp32 (where the keys of a request are
 * split over several workgroups, each part's output is normalised by its own softmax sum and held in half until the
 * parts are merged in fp32).  RANGE: values fed to a GEMM as half operands must stay below 65504 in magnitude; a
 * model with larger normalised activations, attention outputs or SwiGLU products (bf16 would hold them) overflows
 * to infinity there and the layer output turns non-finite: a loud failure, never a finite wrong number.  The layer
 * input / output and the residual stream are bf16 / fp32 and keep bf16's range.
 */

/* Upper bounds that size the context's workspace; step calls beyond them fail with NEXUS_ESHAPE. */
typedef struct {
    int32_t max_prefill_tokens; /* sum of chunk lengths in one prefill sub-batch  */
    int32_t max_prefill_reqs;
    int32_t max_decode_reqs;
    int32_t max_positions;      /* largest absolute position + 1 (rotary table)   */
} nexus_limits;

/*
 * One layer's weights, device bf16, row-major [out_features][in_features]
 * (Eq. 1-3 with each W stored transposed).  w_gate_up holds the ffn gate rows
 * followed by the ffn up rows.  b_qkv may be NULL.  nexus_load_layer() packs
 * them into a library-owned copy; the caller may free its tensors afterwards.
 */
typedef struct {
    const void *attn_norm_g; /* [hidden]                              */
    const void *w_qkv;       /* [(Hq + 2*Hkv)*head_dim][hidden]: q rows, k rows, v rows */
    const void *b_qkv;       /* [(Hq + 2*Hkv)*head_dim] or NULL       */
    const void *w_o;         /* [hidden][Hq*head_dim]                 */
    const void *ffn_norm_g;  /* [hidden]                              */
    const void *w_gate_up;   /* [2*ffn][hidden]                       */
    const void *w_down;      /* [hidden][ffn]                         */
} nexus_layer_weights;

/*
 * Paged KV cache (the paper leaves block management to the serving engine;
 * the caller owns the pools and the page allocator).  Each pool is device
 * memory of n_pages * Hkv * page_size * head_dim bf16 per layer; layer l
 * starts layer_stride_bytes * l after the pool pointer.  The token at
 * position pos of a request lives in page page_table[req][pos / page_size],
 * slot pos % page_size.  The element order INSIDE one (page, kv head) block is
 * private to the library (it is chosen so that the attention kernels read it
 * with full-width coalesced loads); use nexus_kv_import / nexus_kv_export to
 * convert whole pages from / to the canonical order
 * [n_pages][Hkv][page_size][head_dim].  Keys are cached after rotation.
 */
typedef struct {
    void *k_pool, *v_pool;
    int64_t layer_stride_bytes;
    int32_t n_pages;
} nexus_kv_cache;

/*
 * Chunked-prefill sub-batch (Sec. 2.4 / Sec. 3.3: each chunk attends to the KV
 * cached by earlier chunks and appends its own).  Requests are packed along
 * the token axis.  x and y may alias.
 */
typedef struct {
    int32_t n_reqs, n_tokens;    /* host scalars; n_tokens = cu_chunk[n_reqs]                       */
    const void *x;               /* device bf16 [n_tokens][hidden], layer input                     */
    void *y;                     /* device bf16 [n_tokens][hidden], output of the last layer run    */
    const int32_t *cu_chunk;     /* device [n_reqs + 1], exclusive prefix sum of chunk lengths      */
    const int32_t *prefix_len;   /* device [n_reqs], tokens of the request already cached           */
    const int32_t *page_table;   /* device [n_reqs][max_pages]                                      */
    int32_t max_pages;           /* row length of page_table                                        */
    int32_t max_chunk;           /* host hint: >= every chunk length (sizes the launch grids)       */
    int32_t max_total_len;       /* host hint: >= every prefix_len + chunk length                   */
} nexus_prefill_batch;

/*
 * Decode sub-batch (Sec. 2.3: one new token per request against all of its
 * cached KV).  ctx_len[j] counts the tokens cached BEFORE this step: the new
 * token is stored at position ctx_len[j] and attends to ctx_len[j] + 1 keys;
 * the page table row must hold ceil((ctx_len[j] + 1) / page_size) valid pages.
 */
typedef struct {
    int32_t n_reqs;
    const void *x;               /* device bf16 [n_reqs][hidden] */
    void *y;                     /* device bf16 [n_reqs][hidden] */
    const int32_t *ctx_len;      /* device [n_reqs]              */
    const int32_t *page_table;   /* device [n_reqs][max_pages]   */
    int32_t max_pages;
    int32_t max_ctx;             /* host hint: >= every ctx_len[j] + 1 */
} nexus_decode_batch;

/* Filled by nexus_mixed_step when requested (the call then waits for the step to finish). */
typedef struct {
    float t_prefill_ms; /* fork -> prefill chain complete                       */
    float t_decode_ms;  /* fork -> decode chain complete (decode-step latency)  */
    float t_step_ms;    /* fork -> both complete                                */
} nexus_step_timing;

/* Split-selection rule applied to measured latency curves (Sec. 4.1.2 objectives; alpha, beta as in Sec. 5). */
typedef enum {
    NEXUS_POLICY_PREFILL_PRIORITIZED = 0, /* min t_prefill  s.t. t_decode  <= beta  * t_decode(all CUs)  */
    NEXUS_POLICY_DECODE_PRIORITIZED = 1,  /* min t_decode   s.t. t_prefill <= alpha * t_prefill(all CUs) */
    NEXUS_POLICY_MIN_STEP = 2             /* min measured concurrent step time                           */
} nexus_policy;

#define NEXUS_CUS_ALL (-1) /* nexus_set_cu_split(ctx, NEXUS_CUS_ALL, NEXUS_CUS_ALL): unpartitioned, serialized */

/* ---- context ---------------------------------------------------------------------------------------------- */

/* Creates a context on `device` (HIP ordinal): streams, workspace sized by `limits`, rotary table. */
int nexus_create(const nexus_model_desc *desc, const nexus_limits *limits, int device, nexus_ctx **out);
void nexus_destroy(nexus_ctx *ctx);
/* Packs one layer's weights (device pointers) into the library's own tile-ordered copy.  Synchronous: returns when
 * the copy is complete.  The packing runs on a stream of the library's own, which does not wait for any other
 * stream: work that produces the source tensors must have finished before the call. */
int nexus_load_layer(nexus_ctx *ctx, int layer, const nexus_layer_weights *w);
/* Waits for everything the context has enqueued. */
int nexus_sync(nexus_ctx *ctx);
const char *nexus_last_error(void);
/* Number of CUs of the context's GPU (256 on MI355X). */
int nexus_cu_count(nexus_ctx *ctx);

/* ---- KV cache layout conversion (whole pages; device pointers; enqueued on the context's main stream) ------ */

/* canonical bf16 [page_count][Hkv][page_size][head_dim] -> pages [page_begin, page_begin + page_count) of layer */
int nexus_kv_import(nexus_ctx *ctx, const nexus_kv_cache *kv, int layer, const void *k_canon, const void *v_canon,
                    int32_t page_begin, int32_t page_count);
/* the reverse; used by tests to compare appended K/V and untouched slots with the oracle's pools */
int nexus_kv_export(nexus_ctx *ctx, const nexus_kv_cache *kv, int layer, void *k_canon, void *v_canon,
                    int32_t page_begin, int32_t page_count);

/* ---- CU partitioning (Sec. 5: partition layouts are created ahead of use and switched at run time) --------- */

/*
 * Selects the CU share of each phase: prefill_cus + decode_cus <= nexus_cu_count(), both positive multiples of
 * 8.  The chip is eight accelerator dies (XCDs) with an L2 each; every XCD gives each phase the same number of
 * its CUs (a queue's CU mask must keep at least one CU in every XCD, and workgroups are dealt to XCDs
 * round-robin whatever the mask).  Inside an XCD the workgroups are likewise dealt evenly to its 4 shader engines,
 * so a share runs at full speed only when it is a multiple of 32 (4 per XCD); other multiples of 8 are accepted and
 * run at the speed of the next lower multiple of 32.  The two phases then run on two streams whose CU masks are
 * disjoint.  (NEXUS_CUS_ALL, NEXUS_CUS_ALL) selects the unpartitioned layout: one unmasked stream, the mixed step
 * runs prefill then decode back to back (the serialized baseline of Sec. 3.1).
 *
 * A layout (its pair of CU-masked streams) is created the first time its split is selected or prepared (about
 * 10 ms) and kept: selecting it again is a pointer switch on the host (microseconds), waits for nothing and
 * launches nothing (Sec. 4.2: switching must not block the streams).  Work already enqueued on the previous layout
 * keeps running there on its old CU share; each phase's next launch goes to the new layout and is ordered, by
 * events, after the previous launch of the same phase (nexus_mixed_step: of both phases), so for the remainder of
 * a step in flight the old and the new shares may overlap on some CUs.  Up to 8 partitioned layouts stay alive
 * (every split in steps of 32 CUs is 7); selecting a ninth retires the least recently used one, which waits for
 * that layout's work.
 * CU-masked streams are blocking streams in HIP's sense (the call that creates them takes no flags): work issued
 * on the NULL stream waits for them and holds them back.  A caller that overlaps its own copies or kernels with a
 * running phase must issue them on a non-blocking stream.
 */
int nexus_set_cu_split(nexus_ctx *ctx, int prefill_cus, int decode_cus);
/*
 * Creates the layouts of n splits ahead of use (Sec. 5 creates every layout at initialisation) without selecting
 * any: host arrays prefill_cus[n], decode_cus[n], each pair as for nexus_set_cu_split.  Fails with NEXUS_ESHAPE
 * when more partitioned layouts are asked for than are kept alive.
 */
int nexus_prepare_cu_splits(nexus_ctx *ctx, int n, const int32_t *prefill_cus, const int32_t *decode_cus);
/*
 * Destroys every partitioned layout except the current one (waits for their work first); the unpartitioned layout
 * stays.  Every CU-masked stream is a queue of its own, the GPU has fewer hardware queues than a full set of layouts
 * has streams (4 per process by default), and queues beyond that number are time-multiplexed: measured on MI355X, a
 * step whose successor is already enqueued runs 2-3.5 % slower with seven stream pairs alive than with one.  A caller
 * that has settled on a split (after nexus_profile_split, say) gets that back with this call; a caller that keeps
 * switching (Sec. 4.2) keeps the layouts and pays it.
 */
int nexus_retire_cu_splits(nexus_ctx *ctx);

/* ---- the step (layers [layer_begin, layer_end); output of layer l feeds layer l + 1) ----------------------- */

/* Chunked-prefill phase alone, on the prefill stream of the current layout. */
int nexus_prefill_chunk(nexus_ctx *ctx, int layer_begin, int layer_end, const nexus_prefill_batch *pb,
                        const nexus_kv_cache *kv);
/* Decode phase alone, on the decode stream of the current layout. */
int nexus_decode_step(nexus_ctx *ctx, int layer_begin, int layer_end, const nexus_decode_batch *db,
                      const nexus_kv_cache *kv);

/*
 * nexus_decode_step for callers that cannot allocate device memory or let a library do so: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical
 * results; the phase's workspace (activations, split-K partial sums, attention span partials) is laid out in a
 * static device array of the library instead of the context's own buffers, so the call performs no hipMalloc /
 * hipFree and calls no allocating routine; a small clear kernel (no memset node) zeroes what must start at zero.
 * The array is 32 MiB per GPU, exists from library load to process exit and is shared by every context on that
 * GPU: calls that overlap in time on one GPU race on it (calls of one context are ordered by the decode stream).
 * A step whose workspace does not fit fails with NEXUS_ESHAPE before anything is launched: the need grows with
 * n_reqs x (the split-K partial sums of the widest split projection + the attention partials of max_ctx / 256
 * spans); a hidden-4096 GQA layer takes about 23 MB for 64 requests with contexts up to 4096 and does not fit
 * 256 requests with contexts up to 8192.
 * nexus_debug_fetch does not see this call's buffers.
 */
int nexus_decode_step_noalloc(nexus_ctx *ctx, int layer_begin, int layer_end, const nexus_decode_batch *db,
                              const nexus_kv_cache *kv);

/*
 * The step of an engine WITHOUT phase separation (Sec. 2.4, the chunked-prefill engines the paper measures
 * against), for comparison: one batch in which the last n_decode_reqs requests are decode requests written as
 * one-token chunks (chunk length 1, prefix_len = context length, x = the new token's input).  Every projection and
 * norm runs once over all rows, so the weights are read once per step; the chunk rows take the chunked-prefill
 * attention kernel and the decode rows the decode attention kernel.  Runs on the prefill stream of the current
 * layout (select the unpartitioned layout for the baseline proper); output row order = batch row order.
 * max_decode_ctx: largest (context length + 1) among the decode requests.  Limits: the batch within the prefill
 * limits of the context, n_decode_reqs within max_decode_reqs.  Must not overlap a decode phase of the same context
 * (it borrows that phase's attention workspace).
 */
int nexus_fused_step(nexus_ctx *ctx, int layer_begin, int layer_end, const nexus_prefill_batch *batch,
                     int32_t n_decode_reqs, int32_t max_decode_ctx, const nexus_kv_cache *kv);

/*
 * Completion of the last nexus_prefill_chunk / nexus_decode_step of a phase (nexus_phase), without waiting for the
 * other phase: the two calls are asynchronous and, on a partitioned layout, run on different streams, so a caller
 * may keep one loop per phase (Sec. 5) -- launch a phase, poll it, launch its next step -- as long as the two
 * phases touch different requests' pages.  nexus_phase_query returns 1 when that call's work has completed (or
 * none was made), 0 while it is running.  nexus_phase_wait blocks until it has and, if elapsed_ms is not NULL,
 * stores the time between the call's first and last kernel on the GPU's clock.  Both also see a phase launched by
 * nexus_mixed_step or nexus_fused_step (the elapsed time is then reported as -1: those calls bracket the step, not
 * the phase).  A single-phase call is ordered after the previous launch of the same phase on whatever layout that
 * ran, never after the other phase.
 */
int nexus_phase_query(nexus_ctx *ctx, int phase);
int nexus_phase_wait(nexus_ctx *ctx, int phase, float *elapsed_ms);
/*
 * Both phases of one step.  With a partitioned layout they are enqueued on the two CU-masked streams after a
 * common fork event and run concurrently; with the unpartitioned layout they run back to back.  The two
 * sub-batches must touch disjoint requests and pages.  Steps of one context never overlap: each phase starts
 * after the previous launch of BOTH phases of the context (mixed, single-phase or fused), whatever layout that
 * ran on, so the split may be changed between two steps without synchronising.  caller_stream (a hipStream_t) is made to precede the fork
 * and to wait for both phases; with NULL the step is ordered after the context's previous work only, and the
 * caller synchronises with nexus_sync (inputs must be complete when the call is made).  timing may be NULL; when
 * given the call blocks until done.
 */
int nexus_mixed_step(nexus_ctx *ctx, int layer_begin, int layer_end, const nexus_prefill_batch *pb,
                     const nexus_decode_batch *db, const nexus_kv_cache *kv, void *caller_stream,
                     nexus_step_timing *timing);
/*
 * nexus_mixed_step with the decode share handed back to the prefill phase inside the step (Sec. 4.2: the
 * partition follows the load; Sec. 5: a change applies at a kernel boundary and blocks neither stream).  On a
 * partitioned layout the decode step and the prefill layers [layer_begin, handover_layer) run side by side on
 * their shares; the prefill layers [handover_layer, layer_end) are launched on the unmasked stream and so run on
 * every CU, ordered after the layers before them by an event.  They do not wait for the decode step: when
 * handover_layer is chosen so that the decode step has finished by then (from the phase times nexus_profile_split
 * measures), the CUs it held are not idle for the rest of the step; when it has not, the two share CUs until it
 * has.  Results are bit-identical to nexus_mixed_step for every handover_layer (no summation order depends on the
 * CU share).  handover_layer = layer_end, or the unpartitioned layout, is nexus_mixed_step itself.  Everything else
 * (ordering against other steps, caller_stream, timing) as there; t_prefill_ms spans both parts.
 * NEXUS_EINVAL when handover_layer is outside [layer_begin, layer_end].
 *
 * handover_layer = NEXUS_HANDOVER_AUTO lets the library choose: every such step is bracketed by events, and once a
 * step has completed its times are read back (without waiting: a step still running is skipped and read later) --
 * how long the decode step took next to the prefill phase, and how long a prefill layer took on the share.  The next
 * automatic step on the same layout hands over at the first layer boundary after the decode step's expected end (at
 * least one layer runs on the share); the first automatic step on a layout has no measurement and holds the split to
 * the end of the step, which yields one.  The choice follows the load from step to step (Sec. 4.2) at the price of
 * four event records per step.  nexus_last_handover_layer returns the layer the most recent mixed step handed over
 * at (layer_end when it did not; 0 before the first step).
 */
#define NEXUS_HANDOVER_AUTO (-1)
int nexus_mixed_step_handover(nexus_ctx *ctx, int layer_begin, int layer_end, int handover_layer,
                              const nexus_prefill_batch *pb, const nexus_decode_batch *db, const nexus_kv_cache *kv,
                              void *caller_stream, nexus_step_timing *timing);
int nexus_last_handover_layer(nexus_ctx *ctx);
/*
 * Latency-vs-CUs profiling (Sec. 3.2) and split choice (Sec. 4.1.2 on measured curves).  For each candidate i,
 * prefill gets cand_prefill_cus[i] CUs and decode the remaining ones; the phases are timed alone (median of
 * `repeats` runs after one warm-up) and together.  Host output arrays have n_cand entries; t_alone_all_ms[2]
 * receives each phase alone on the whole GPU.  The chosen layout is left active.  KV pools are overwritten at
 * the appended positions only (re-running a step rewrites the same slots with the same values).
 */
int nexus_profile_split(nexus_ctx *ctx, int layer_begin, int layer_end, const nexus_prefill_batch *pb,
                        const nexus_decode_batch *db, const nexus_kv_cache *kv, const int32_t *cand_prefill_cus,
                        int n_cand, int policy, float alpha, float beta, int repeats, float *t_prefill_ms,
                        float *t_decode_ms, float *t_step_ms, float *t_alone_all_ms, int32_t *chosen_prefill_cus);

/*
 * The selection rule of nexus_profile_split on its own (host only, no GPU work): returns the index of the chosen
 * candidate given the measured curves, or a negative status.  When no candidate meets the slack the one that
 * violates it least is taken; ties go to the lower index.
 */
int nexus_choose_split(int n_cand, const float *t_prefill_ms, const float *t_decode_ms, const float *t_step_ms,
                       float t_prefill_all_ms, float t_decode_all_ms, int policy, float alpha, float beta);

/* ---- partition controller: cost model, objectives, greedy search, buffer zone (host only, no GPU work) ------ */

/*
 * One operator of a phase for the latency model of Sec. 4.1.1: its compute time on a share r of the GPU is
 * flops / (r C) up to the saturation share r_sat and flops / (r_sat C) * (1 + lambda (r - r_sat)) beyond it
 * (Eq. 7); its memory time is bytes / B.  kind tells the contention model which traffic is attention (Eq. 8-9).
 */
typedef enum { NEXUS_OP_DENSE = 0, NEXUS_OP_ATTENTION = 1 } nexus_op_kind;
typedef struct {
    double flops, bytes; /* per iteration of the phase (all layers) */
    double r_sat;        /* in (0, 1] */
    double lambda;
    int32_t kind;        /* nexus_op_kind */
    int32_t reserved;
} nexus_cost_op;
typedef struct {
    double peak_flops;       /* C */
    double peak_bytes_per_s; /* B */
    int32_t n_prefill_ops, n_decode_ops;
    const nexus_cost_op *prefill_ops, *decode_ops; /* host arrays, caller-owned */
} nexus_cost_model;

/*
 * CostModel(phase, R) of Alg. 1: latency in seconds of `phase` on `share` of `total` equal steps of the GPU while
 * the other phase holds the rest; a phase is the sum over its operators of max(compute time, memory time)
 * (Eq. 5-6).  Decode attention moves its bytes at the bandwidth left by prefill: with P_attn the fraction of
 * prefill's time spent in attention (Eq. 8), decode gets m_d / (m_d + m_p1) of B during it and m_d / (m_d + m_p2)
 * otherwise (m_d, m_p1, m_p2: bytes of decode attention, prefill attention, prefill dense operators), Eq. 9.
 * At share == total the other phase is taken at its floor of one step for the contention term (Alg. 1 reads its
 * reference latency from this same function at R = 100, where Eq. 8 has no value; a model whose other phase has
 * no operators has no contention at any share).  1 <= share <= total, else NEXUS_EINVAL.
 */
int nexus_cost_latency(const nexus_cost_model *model, int phase, int share, int total, double *seconds);

/*
 * AdjustPartition of Alg. 1 for the prioritised `target_phase`: starting from the current split, the target gives
 * up steps until the other phase's modelled latency is within its budget (alpha x prefill's, beta x decode's
 * latency on every step of the GPU as nexus_cost_latency gives it, Sec. 4.1.2), then takes steps back while the
 * budget still holds.  Both phases
 * keep at least one step.  Outputs: the new prefill share and (if non-null) the number of model evaluations.
 */
int nexus_adjust_partition(const nexus_cost_model *model, int target_phase, int cur_prefill_share, int total,
                           double alpha, double beta, int32_t *new_prefill_share, int32_t *evaluations);

/*
 * PartitionController of Alg. 1: decode is prioritised when kv_usage > kv_switch, prefill otherwise (Sec. 4.1.2,
 * runtime switching); a change of fewer than `delta` steps is suppressed (the buffer zone of Sec. 4.2).
 */
int nexus_partition_controller(const nexus_cost_model *model, double kv_usage, double kv_switch,
                               int cur_prefill_share, int total, double alpha, double beta, int delta,
                               int32_t *new_prefill_share);

/*
 * Extracts an operator's curve parameters from n measured (share in (0, 1], seconds) points (Sec. 4.1.1: R_sat
 * and lambda come from measurements under varying allocations; the paper does not say how): each measured share
 * is tried as R_sat, the effective work is the mean of t r C at or below it, lambda the least-squares slope of
 * t / t_sat - 1 above it; the candidate with the smallest squared relative error is returned.  n >= 1.
 */
int nexus_cost_fit(int n, const double *shares, const double *seconds, double peak_flops, double *flops,
                   double *r_sat, double *lambda);

/*
 * Algorithmic flops and bytes of the five operators of each phase (order: QKV, attention, O, gate/up, down) for
 * `layers` layers of `desc`, from the quantities the controller sees (Fig. 6): prefill_tokens = P_T and the
 * (query, visible key) pairs of its attention, prefill_kv_tokens = KV_p (tokens whose K/V the chunk reads),
 * decode_reqs = B_d, decode_kv_tokens = KV_d.  Dense operators move their weights once, attention the K/V it
 * reads.  r_sat is set to 1 and lambda to 0; nexus_cost_fit refines them.  Both arrays have 5 entries.
 */
int nexus_cost_describe(const nexus_model_desc *desc, int layers, double prefill_tokens, double prefill_pairs,
                        double prefill_kv_tokens, double decode_reqs, double decode_kv_tokens,
                        nexus_cost_op *prefill_ops, nexus_cost_op *decode_ops);

/* ---- phase-specific schedulers and the iteration loop around them (Sec. 4.3, Alg. 2; host only) ---------- */

/*
 * The prefill queue is ordered either by arrival (FCFS) or by Shortest Prompt First with the age term of Eq. 10:
 * score = remaining prompt tokens - gamma * (now - arrival), lowest first, ties to the earlier arrival, then to the
 * lower id.  Requests are taken in that order while the batch's tokens stay within token_budget (Alg. 2); the
 * first request that does not fit ends the batch, after taking what is left of the budget as a partial chunk when
 * chunk_tail is set (chunked prefill, Sec. 5; without it a prompt longer than the budget is never scheduled).
 * Decode is FCFS (Sec. 4.3.2): a request whose last prompt chunk has committed has emitted its first token and
 * joins the decode pool, in the order of those commits, as soon as the pool has room; every pool member decodes
 * one token per iteration until it has emitted output_len tokens.
 * KV pages: a request is admitted to its first chunk only when the pages of its whole lifetime
 * (prompt_len + output_len - 1 tokens) can be reserved; a request that cannot holds back the not yet admitted
 * requests behind it, never the admitted ones.  Pages are taken from a free list as positions get written and go
 * back when the request finishes.
 */
typedef struct nexus_sched nexus_sched;
typedef enum { NEXUS_PREFILL_FCFS = 0, NEXUS_PREFILL_SPF = 1 } nexus_prefill_policy;
typedef struct {
    int32_t prefill_policy;   /* nexus_prefill_policy                                             */
    int32_t token_budget;     /* B of Alg. 2: prompt tokens per iteration                         */
    int32_t max_prefill_reqs; /* requests per prefill batch; 0 = no limit                         */
    int32_t max_decode_reqs;  /* capacity of the decode pool                                      */
    int32_t page_size, n_pages;
    int32_t chunk_tail;       /* see above; 1 for chunked prefill                                 */
    int32_t reserved;         /* must be 0                                                        */
    double gamma;             /* tokens per second of age (Sec. 5 uses 15)                        */
    const int32_t *page_order; /* host, a permutation of 0..n_pages-1: the order in which the free list first hands
                                  pages out; NULL for 0, 1, 2, ...  Copied by nexus_sched_create.  */
} nexus_sched_config;

/*
 * The batches of one iteration.  All pointers are host memory owned by the scheduler, valid until its next call.
 * Page tables are [n][max_pages] row-major, -1 past a request's own pages; a request holds exactly the pages
 * covering the positions it will have written when the iteration commits.  The fields map one to one onto
 * nexus_prefill_batch / nexus_decode_batch.
 */
typedef struct {
    int32_t n_prefill, prefill_tokens;
    const int32_t *prefill_req;        /* [n_prefill] request ids                           */
    const int32_t *prefill_prefix;     /* [n_prefill] tokens already cached                 */
    const int32_t *prefill_chunk;      /* [n_prefill] tokens of this chunk                  */
    const int32_t *prefill_cu_chunk;   /* [n_prefill + 1] exclusive prefix sum of the above */
    const int32_t *prefill_page_table;
    int32_t prefill_max_pages, prefill_max_chunk, prefill_max_total_len;
    int32_t n_decode;
    const int32_t *decode_req;         /* [n_decode] request ids, in pool order             */
    const int32_t *decode_ctx;         /* [n_decode] tokens cached before the step          */
    const int32_t *decode_page_table;
    int32_t decode_max_pages, decode_max_ctx;
    int32_t kv_used_pages, kv_total_pages; /* pages holding tokens / pool size: KV_u of Alg. 1 */
} nexus_sched_batch;

typedef struct {
    double arrival_s, first_token_s, finish_s; /* -1 while not reached */
    int32_t prompt_len, output_len, prefilled, emitted, n_pages, state; /* state: 0 waiting, 1 ready, 2 decoding, 3 done */
} nexus_sched_request_info;

/* Serving metrics of Sec. 6.1 over what has been committed so far; percentiles are nearest-rank. */
typedef struct {
    int32_t n_submitted, n_first_token, n_finished, reserved;
    int64_t prefill_tokens, decode_tokens;
    double ttft_mean, ttft_p50, ttft_p95, ttft_p99, ttft_max;          /* first token - arrival              */
    double tbt_mean, tbt_p50, tbt_p95, tbt_p99, tbt_max;               /* between consecutive tokens         */
    double norm_latency_mean, norm_latency_p95;                        /* (finish - arrival) / output tokens */
} nexus_sched_summary;

int nexus_sched_create(const nexus_sched_config *cfg, nexus_sched **out);
void nexus_sched_destroy(nexus_sched *s);
/* Queues a request (arrival in seconds on the caller's clock; prompt_len, output_len >= 1).  Fails with
 * NEXUS_ESHAPE when the request's lifetime needs more pages than the pool has. */
int nexus_sched_submit(nexus_sched *s, double arrival_s, int32_t prompt_len, int32_t output_len, int32_t *id_out);
/* Forms the batches of the iteration starting at now_s from the requests with arrival <= now_s.  Either batch may
 * be empty.  Must be followed by nexus_sched_commit before the next call. */
int nexus_sched_next(nexus_sched *s, double now_s, nexus_sched_batch *out);
/* The iteration formed by the last nexus_sched_next completed at end_s (>= its now_s). */
int nexus_sched_commit(nexus_sched *s, double end_s);
/*
 * The two phases may also tick independently (Sec. 5 runs them as separate loops): nexus_sched_next_phase forms the
 * batch of one phase (nexus_phase) and fills that phase's fields of *out (the other phase's are zeroed),
 * nexus_sched_commit_phase completes it.  At most one tick per phase is open at a time; an empty batch opens none
 * and needs no commit.  A request that completes its prompt at a prefill commit joins the pool at the next decode
 * tick.  Not to be mixed with an open coupled iteration (NEXUS_ESTATE).
 */
int nexus_sched_next_phase(nexus_sched *s, int phase, double now_s, nexus_sched_batch *out);
int nexus_sched_commit_phase(nexus_sched *s, int phase, double end_s);
int nexus_sched_request(const nexus_sched *s, int32_t id, nexus_sched_request_info *out);
int nexus_sched_summarize(const nexus_sched *s, nexus_sched_summary *out);
/* Raw samples: kind 0 = TTFT (by request id), 1 = TBT (in commit order), 2 = normalised latency (by request id).
 * Writes up to cap doubles to host `out` (may be NULL with cap 0) and the total number available to *n. */
int nexus_sched_samples(const nexus_sched *s, int kind, double *out, int32_t cap, int32_t *n);

/* ---- validation of device-side integer inputs (debug mode) ------------------------------------------------ */

/*
 * on != 0: every step call (prefill chunk, decode step, mixed step, fused step) first copies its chunk offsets,
 * prefix / context lengths and page tables to the host, waits for the copy, and checks them with
 * nexus_validate_batches against the KV cache it was given; a violation fails the call with NEXUS_EINVAL before
 * anything is launched.  The arrays must be complete when the call is made.  Costs a device-to-host round trip
 * per step: a debugging aid, off by default (or NEXUS_DEBUG_CHECKS=1 in the environment at nexus_create).
 */
int nexus_set_debug_checks(nexus_ctx *ctx, int on);
/*
 * The check itself, host only (every pointer is HOST memory; a batch with zero requests is absent and its pointers
 * may be NULL): chunk offsets are an exclusive prefix sum ending at n_prefill_tokens; lengths are non-negative and
 * within max_chunk / max_total_len / max_ctx; every page a request touches (positions [0, prefix + chunk) or
 * [0, ctx + 1)) lies in [0, n_pages) and inside its table row; a page that one request writes (the pages of the
 * positions it appends) is touched by no other request of the step.  Returns NEXUS_OK or NEXUS_EINVAL with the
 * offending request and entry in nexus_last_error().
 */
int nexus_validate_batches(int32_t n_pages, int32_t page_size, int32_t n_prefill_reqs, int32_t n_prefill_tokens,
                           const int32_t *cu_chunk, const int32_t *prefix_len, const int32_t *prefill_page_table,
                           int32_t prefill_max_pages, int32_t max_chunk, int32_t max_total_len, int32_t n_decode_reqs,
                           const int32_t *ctx_len, const int32_t *decode_page_table, int32_t decode_max_pages, int32_t max_ctx);

/* ---- measurement and test hooks ----------------------------------------------------------------------------- */

/* Kernel ids for nexus_trace_*: one per kernel family on the path. */
typedef enum {
    NEXUS_K_RMSNORM = 0, NEXUS_K_GEMM_QKV, NEXUS_K_ROPE_APPEND, NEXUS_K_ATTN_PREFILL, NEXUS_K_GEMM_O,
    NEXUS_K_GEMM_GATE_UP, NEXUS_K_GEMM_DOWN, NEXUS_K_ATTN_DECODE, NEXUS_K_ATTN_MERGE, NEXUS_K_SPLITK_REDUCE,
    NEXUS_K_COUNT
} nexus_kernel_id;
typedef enum { NEXUS_PHASE_PREFILL = 0, NEXUS_PHASE_DECODE = 1 } nexus_phase;

/*
 * While tracing is on, every launch of (phase, kernel) is bracketed by HIP events on the stream it runs on.
 * nexus_trace_read waits, returns the mean duration in milliseconds and the number of launches seen since
 * nexus_trace_begin, and turns tracing off.  At most 4096 launches are recorded.
 */
int nexus_trace_begin(nexus_ctx *ctx, int phase, int kernel);
int nexus_trace_read(nexus_ctx *ctx, float *mean_ms, int32_t *launches);

/* Intermediate buffers of the last step of a phase, converted to row-major fp32 (device out pointer). */
typedef enum {
    NEXUS_BUF_NORM1 = 0, /* [T][hidden]   RMSNorm output feeding the QKV projection */
    NEXUS_BUF_Q,         /* [T][Hq*hd]    rotated queries                           */
    NEXUS_BUF_ATTN,      /* [T][Hq*hd]    attention output                          */
    NEXUS_BUF_X1,        /* [T][hidden]   residual stream after attention           */
    NEXUS_BUF_ACT        /* [T][ffn]      SwiGLU activation feeding the down projection */
} nexus_debug_buf;
int nexus_debug_fetch(nexus_ctx *ctx, int phase, int which, int32_t n_tokens, void *out);

/*
 * Runs a probe kernel of n_blocks one-wave workgroups on the stream of `phase` in the current layout and
 * returns, per hardware (XCD, shader engine, CU), how many workgroups ran there: host out_counts[8 * 128] int32,
 * index xcd * 128 + shader_engine * 16 + cu, from the wave's hardware-id registers.
 */
int nexus_debug_cu_probe(nexus_ctx *ctx, int phase, int n_blocks, int32_t *out_counts);

/*
 * The order in which the token-per-workgroup kernels (RMSNorm, rotary + append) visit the n tokens of a batch:
 * workgroup b handles token nexus_debug_token_order(b, n) (the long-batch RMSNorm, four tokens per workgroup, applies
 * it to its groups of four).  Workgroups are dealt to the 8 XCDs round-robin and
 * neighbouring tokens share cache lines in what those kernels write, so inside every aligned group of 256 (64)
 * workgroups the workgroups of one XCD take 32 (8) consecutive tokens; a tail that fills no whole group keeps its
 * order.  A permutation of [0, n) for every n.  Host only; returns a negative status for b outside [0, n).
 */
int nexus_debug_token_order(int b, int n);

#ifdef __cplusplus
}
#endif
#endif /* NEXUS_H */
