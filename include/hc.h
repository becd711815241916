/* hc.h -- C ABI of the HeteroCache decode hot path for AMD MI355X (gfx950).
 *
 * What is computed is the per-step online inference of HeteroCache (arXiv 2601.13684,
 * Sec. 4.3 "Hierarchical Storage & Retrieval" and Algorithm 1, stage 3), for one layer:
 *
 *   hc_decode_attn      attention of the decode token over the heterogeneous cache C_GPU:
 *                       full (volatile / pivot) heads over the whole context, compressed
 *                       (anchor / satellite) heads over their l_i resident slots;
 *   hc_rep_topk_drift   the pivot heads' drift monitor: GQA-aggregated score (App. C.1),
 *                       TopIndices_k, overlap with the baseline set (Eq. 9), windowed-median
 *                       retrieval signal (Eq. 10), baseline update;
 *   hc_gather_retrieve  AsyncUpdate: C_GPU^(s) <- C_CPU^(s)[I_s] for the satellites of every
 *                       pivot whose signal fired, reading a pinned host-memory tier.
 *
 * Conventions
 *   - C99, no C++ types.  Every function returns an hc_status; nothing aborts, throws or prints.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers ordinary host memory,
 *     "pinned" pointers host memory allocated with hipHostMalloc (device-visible).
 *   - The caller owns every buffer it passes in.  The library owns only what hc_create and
 *     hc_layer_create allocate (split-K partials, selection workspaces, launch plans) and
 *     frees it in the matching destroy call.  No caller pointer is kept after a call returns.
 *   - The three hot-path calls only enqueue work on the given HIP stream: they never
 *     synchronise, allocate or copy from the host, so they may be captured in a HIP graph.
 *     Results are valid once the stream (or done_event) has completed.  Trigger decisions
 *     stay in device memory (flag); the host may read them later.
 *   - One hc_ctx per host thread; calls on one ctx are not re-entrant, and two hot-path calls
 *     that use the same workspace (two hc_decode_attn, or two hc_rep_topk_drift) must be
 *     ordered by the caller's streams.  A decode_attn and a rep_topk_drift may overlap.
 *   - Arguments are validated on the host before anything is launched.
 *
 * Index-list tables (topk_idx, base_idx) have one row of max_k int32 per (b, KV head):
 * row (b*Hkv + h).  Per-head scalars (inter, flag) are indexed the same way; ring has
 * (window + 1) int32 per row: [0] = number of stored values, [1..] = values, oldest first.
 */
#ifndef HC_H
#define HC_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hc_ctx hc_ctx;       /* device-wide workspaces                                  */
typedef struct hc_layer hc_layer;   /* one layer's head table, split-K plan and selection plan */

typedef enum {
    HC_OK = 0,
    HC_EINVAL = 1,   /* null pointer, bad enum, inconsistent role / rep table                   */
    HC_ESHAPE = 2,   /* a size is outside what the kernels support                              */
    HC_ENOMEM = 3,   /* host or device allocation failed                                        */
    HC_EHIP = 4,     /* a HIP call failed; hc_last_error has its text                           */
    HC_ESTATE = 5    /* object used after destroy / with the wrong ctx                          */
} hc_status;

enum { HC_ROLE_FULL = 0, HC_ROLE_SATELLITE = 1, HC_ROLE_ANCHOR = 2 };
enum { HC_METRIC_OVERLAP = 0, HC_METRIC_JACCARD = 1 };
enum { HC_AGG_PROB = 0, HC_AGG_LOGIT = 1 };
enum { HC_WINDOW_SLIDING = 0, HC_WINDOW_TUMBLING = 1, HC_WINDOW_RESCORED = 2 };
enum { HC_MAX_WINDOW = 64, HC_MAX_K_PER_REP = 8, HC_MAX_GROUP = 8 };
enum { HC_STATIC_MAX_PARTIALS = 1024 };   /* largest split-K plan hc_decode_attn_static accepts */

typedef struct {
    int32_t B;         /* sequences in the batch (>= 1)                                         */
    int32_t Hq;        /* query heads; Hq = G * Hkv with G in {1, 2, 4, 8}                      */
    int32_t Hkv;       /* KV heads                                                              */
    int32_t D;         /* head dimension; must be 128                                           */
    int32_t max_ctx;   /* upper bound of every context length; multiple of 64; row stride of
                          rep_logits and scores                                                 */
    int32_t max_k;     /* row stride of the index-list tables; >= every k used                  */
    int32_t window;    /* W of Eq. 10, 1..HC_MAX_WINDOW                                         */
    int32_t metric;    /* HC_METRIC_OVERLAP: inter/k (Eq. 9); HC_METRIC_JACCARD: inter/(2k-inter) */
    int32_t tau_num;   /* drift threshold tau_drift = tau_num / tau_den, compared exactly in    */
    int32_t tau_den;   /*   integers: statistic < tau  (strict, Eq. 10); tau_den >= 1           */
    int32_t agg;       /* HC_AGG_PROB: mean over the GQA group of softmax weights (App. C.1);
                          HC_AGG_LOGIT: mean of scaled logits (exactly reproducible test mode)  */
    int32_t window_mode; /* HC_WINDOW_SLIDING: Eq. 10 as written, tested at every step once W overlaps are
                          stored, the store emptied on a retrieval.  HC_WINDOW_TUMBLING: Algorithm 1's
                          loop, tested when t mod W = 0 over the W steps since the last test, the store
                          emptied after every test.  (Algorithm 1 re-scores the W buffered queries at
                          that point; as long as the pivot's cache has not changed in between, that
                          gives the overlaps already computed at those steps, which are what is
                          stored.)  HC_WINDOW_RESCORED: the same loop with that re-scoring done:
                          hc_rescore_window, called before the monitor at every step, buffers the
                          queries and at the test step replaces the stored overlaps of the window's
                          earlier queries by those of their top-k over the pivot's cache as it is
                          then (they differ once the context grows inside a window).             */
} hc_config;

/* One KV head of one sequence; table of B*Hkv entries, row (b*Hkv + h), HOST memory. */
typedef struct {
    int64_t k_off;     /* element (bf16) offset of this head's K rows [len][D] in the arena ([cap][D]
                          for a full head that may grow); multiple of 8                          */
    int64_t v_off;     /* same for V rows                                                        */
    int64_t tier_off;  /* satellites: element offset of this head's [ctx][2][D] block (K row then
                          V row per position; [cap][2][D] if it may grow) in the host tier;
                          multiple of 8; others: ignored                                         */
    int32_t ctx;       /* N_b: context length of the sequence, 1..max_ctx                        */
    int32_t len;       /* resident rows: ctx for a full head, the budget l_i for a compressed one */
    int32_t role;      /* HC_ROLE_*                                                              */
    int32_t rep;       /* satellite: KV-head index (same sequence) of its pivot, which must be
                          HC_ROLE_FULL; otherwise -1                                             */
    int32_t sink;      /* compressed: slots [0,sink) hold positions [0,sink)                     */
    int32_t recent;    /* compressed: slots [sink,sink+recent) hold positions [ctx-recent,ctx);
                          slots [sink+recent, len) are the r retrieved ones                      */
    int32_t k_mon;     /* pivot: size of the monitored set (L_base of Eq. 9); 0 = largest r of
                          its satellites                                                         */
    int32_t cap;       /* room to grow (hc_append_kv): rows that this head's K block, V block (full heads)
                          and host-tier block (satellites) are laid out for; 0 = none (len resp. ctx);
                          otherwise ctx <= cap <= max_ctx.  Compressed heads' K/V blocks stay [len][D]  */
} hc_head_desc;

/* ---- life cycle (these may allocate and synchronise; not for capture) -------------------- */
hc_status hc_create(const hc_config* cfg, hc_ctx** out);
hc_status hc_destroy(hc_ctx* ctx);
const char* hc_strerror(hc_status st);
const char* hc_last_error(const hc_ctx* ctx);       /* text of the last failure on this ctx   */

/* Validates the head table (all satellites of one pivot must share sink and recent; every k
 * must fit the candidate range [sink, ctx-recent) and max_k; at most HC_MAX_K_PER_REP distinct
 * set sizes per pivot), builds the split-K work partition and uploads the plans. */
hc_status hc_layer_create(hc_ctx* ctx, const hc_head_desc* heads_host, hc_layer** out);
hc_status hc_layer_destroy(hc_layer* layer);
/* Number of pivots (full heads with at least one satellite), and the slot 0..n-1 of pivot (b,h)
 * in rep_logits / scores (-1 if (b,h) is not a pivot). */
int32_t hc_layer_num_reps(const hc_layer* layer);
int32_t hc_layer_rep_slot(const hc_layer* layer, int32_t b, int32_t h);
/* Split-K plan facts for reporting: workgroups launched and partial results combined. */
int32_t hc_layer_num_workgroups(const hc_layer* layer);
int32_t hc_layer_num_partials(const hc_layer* layer);
/* Tuning knob (before hc_layer_create): target workgroups per compute unit of the split pass
 * (default 2) and host override of the compute-unit count (0 = ask the device). */
hc_status hc_set_split(hc_ctx* ctx, int32_t workgroups_per_cu, int32_t compute_units);
/* Tuning knob (before hc_layer_create): relative size of the share of rows that a workgroup of the
 * split pass gets, by the die it runs on (workgroup index mod 8) and its dispatch slot (first or
 * second half of the indices): weights16[die * 2 + slot], each in 0.25..4; NULL restores the built-in
 * defaults (measured on MI355X: the second workgroup on a compute unit and the workgroups on odd
 * dies stream a few per cent slower).  Used when the number of workgroups is a multiple of 16. */
hc_status hc_set_share_weights(hc_ctx* ctx, const float* weights16);
/* Copies the 16 weights in use (built-in, set, or measured by hc_layer_tune) to host memory weights16. */
hc_status hc_get_share_weights(const hc_ctx* ctx, float* weights16);

/* Measures the share weights (see hc_set_share_weights) on the device at hand: runs the layer's split pass
 * 18 times per round with per-workgroup timestamps (out, lse and rep_logits are overwritten with the
 * results of attention for q, as hc_decode_attn would), equalises the mean finish times of the 16 (die,
 * dispatch slot) classes, replans the layer, and leaves the weights in the context for layers created
 * later.  Which dies stream slower differs between devices; the built-in weights are one device's.
 * Set-up time only: allocates, synchronises the stream.  A plan whose shares are not weighted (short
 * passes) is left alone.  rounds: 1..16; 4 is enough. */
hc_status hc_layer_tune(hc_ctx* ctx, hc_layer* layer, const void* kv_arena, const void* q, float* out, float* lse,
                        float* rep_logits, int32_t rounds, void* stream);

/* Tuning knob: how many 1024-candidate chunks a workgroup of the monitor's selection passes takes
 * (1..64); 0 (default) lets every call choose: 1 for a single layer (many small workgroups, lowest
 * latency), up to 8 for a batch of layers (histograms cleared and flushed once per workgroup). */
hc_status hc_set_monitor_span(hc_ctx* ctx, int32_t span);

/* The pivot-logit filter (before hc_layer_create; layers created while it is on carry its buffers).  margin 0
 * (default): off.  margin >= 1: hc_decode_attn / hc_decode_step store, of a pivot's scaled logits, only the rows
 * that can matter to the monitor, and hc_rep_topk_drift works over those rows.  The 7 MB of logits per 224K pivot
 * that the monitor otherwise writes and reads beside the attention pass shrink to a few hundred KB.
 *   How: after every decision the monitor leaves, per pivot, this step's log-sum-exp and cut = (smallest score
 *   that made it into any of the pivot's lists) / margin.  The next step's split pass keeps position j of the
 *   candidate range only if (1/G) sum_g exp(logit_g[j] - lse_prev_g) >= cut.  The monitor then scores the kept
 *   rows with the step's own log-sum-exp, selects among them, and CHECKS that the smallest list threshold it
 *   found is at least cut * max_g exp(lse_prev_g - lse_g) (with room for rounding): every dropped row's true
 *   score lies below that bound, so none can belong to any list, and the lists, the overlap and the decision
 *   are exactly those of the unfiltered monitor.  If the check fails (or fewer rows were kept than the longest
 *   list needs, or more than a few times that), all of the pivot's logits are computed again, with the same
 *   arithmetic as the split pass, and the plain passes redo that pivot: the same results, a slower step.  All of
 *   this is decided on the device; the calls stay enqueue-only.  The first step (no filter set yet) keeps every row.
 *   margin trades kept rows against fallbacks: 1.25 keeps about 1.6 times the longest list at a 224K context and
 *   has not fallen back on the synthetic workloads; a query whose attention changes abruptly needs more.
 *   What changes for the caller: rep_logits and scores then hold the kept rows only (scores[p][0, n): the scores
 *   of the n kept rows in position order; hc_layer_filter_view gives their positions), except for a pivot that
 *   fell back, whose rows of both are dense as without the filter; the layer remembers the kv_arena of its last
 *   attention call (the fallback reads K from it) and keeps its own copy of the pivots' queries.  Only with
 *   HC_AGG_PROB; with HC_AGG_LOGIT, given scores, the window's re-scored queries and the prefill-time selection
 *   the plain passes run.
 *   min_candidates: only layers in which some pivot has at least this many candidate positions filter.  The filtered
 *   monitor costs more launches per call (the stand-by passes are enqueued whether or not they find work), which a
 *   short context does not earn back: measured on MI355X, filtering pays from about 64K candidates per pivot. */
hc_status hc_set_logit_filter(hc_ctx* ctx, float margin, int32_t min_candidates);
/* Per-pivot counters of the monitor since the layer was created, copied to host memory (synchronous):
 * counts4[0] decisions taken (windows tested), [1] retrievals triggered, [2] steps decided by the dense fallback of
 * the filter, [3] rows the filter kept at the last step (0xffffffff: the last step was not filtered). */
hc_status hc_layer_monitor_counts(const hc_layer* layer, int32_t b, int32_t h, uint32_t* counts4);
/* Device pointers into a filtering layer's state, for inspection (NULL if the layer does not filter):
 * kept_pos [num_reps][max_ctx] int32, the positions of the rows kept at the last step, ascending, the scores of
 * which are scores[p][0, n); fell_back [num_reps] int32, != 0 where the last step's check failed. */
hc_status hc_layer_filter_view(const hc_layer* layer, const int32_t** kept_pos, const int32_t** fell_back);

/* Tuning knob: launch shape of the gather kernel: at most `workgroups` workgroups (1..4096) of `threads` threads (64,
 * 128 or 256); a workgroup has threads / 8 positions in flight.  Default 96 x 256.  What matters is how the host
 * reads, which take microseconds each, are spread over the compute units: the attention pass's loads on a unit queue
 * behind them. */
hc_status hc_set_gather_shape(hc_ctx* ctx, int32_t workgroups, int32_t threads);

/* Tuning knob: how much LDS every workgroup that hc_decode_step launches on its side stream reserves (bytes: 80 KB + 1
 * .. 100 KB, default 81 KB; or 0: only what the kernels need).  More than half of a compute unit's LDS means that a
 * compute unit never holds two workgroups of the side stream at once, so that, whichever stream's kernel gets to an
 * idle compute unit first, the two workgroups of the attention pass still find their registers, wave slots and LDS
 * there: an attention workgroup that has to wait for a place delays its whole launch.  The price: a side-stream
 * kernel with more workgroups than compute units runs in several rounds (the filtered monitor's launches are sized
 * for about twice the longest list, not for the context, to stay below that).  Measured: -1.1 % of the step at the
 * 224K workload, -1.5 % with 16 ragged sequences, no change at 128K with refills at most steps.  Applies to groups of
 * layers whose attention passes all filter the pivot logits (hc_set_logit_filter): only that form of the split pass
 * is small enough (25 KB of LDS per workgroup) to fit twice beside such a reservation. */
hc_status hc_set_side_lds(hc_ctx* ctx, int32_t bytes);

/* Measurement hook: hands the library n pairs of hipEvent_t (host arrays of handles, copied).  The
 * next n launches of the split-pass kernel, from hc_decode_attn or hc_decode_step, attach pair i to
 * their i-th dispatch, so that hipEventElapsedTime(ev_begin[i], ev_end[i]) is that kernel's execution
 * time alone, as a profiler's kernel trace reports it.  After n launches, or with n = 0, no events
 * are recorded.  The events are the caller's; they are only recorded, never waited on or destroyed. */
hc_status hc_set_timing_events(hc_ctx* ctx, void* const* ev_begin, void* const* ev_end, int32_t n);

/* Measurement helpers: two plain streaming kernels that compute nothing of the method and only show what the
 * machine at hand gives the kernels they bound.  hc_probe_stream_read reads `bytes` (a multiple of 16 is read)
 * of device memory once with coalesced 16-byte loads (streaming != 0: marked non-temporal, as the attention pass
 * marks its K/V loads) from `workgroups` workgroups of 256 threads (2048 is a good choice) and stores nothing
 * (dev_sink: 4 bytes of device memory or NULL): its rate is the read
 * bandwidth of HBM that a kernel can reach, the bound of the attention pass.  hc_probe_host_copy copies `bytes`
 * from pinned host memory to device memory with a kernel that reads the host memory over the host link, as the
 * gather reads the host tier: its rate is the gather's bound.  Enqueue-only; the caller times them. */
hc_status hc_probe_stream_read(const void* dev_buf, size_t bytes, void* dev_sink, int32_t workgroups, int32_t streaming,
                               void* stream);
hc_status hc_probe_host_copy(const void* pinned_src, void* dev_dst, size_t bytes, int32_t workgroups, void* stream);

/* Host-only dry run of hc_layer_create: validates the head table exactly as hc_layer_create does
 * and reports the plan it would build for a device with the given number of compute units.  Touches
 * no GPU.  err (may be NULL) receives the text of a validation failure. */
typedef struct {
    int32_t n_workgroups;             /* workgroups of the split pass                               */
    int32_t n_partials;               /* partial results the combine pass merges                    */
    int32_t n_reps;                   /* pivots                                                     */
    int32_t n_lists;                  /* index lists emitted per monitor call                       */
    int32_t n_satellites;             /* satellites with at least one retrieved slot                */
    int32_t max_rows_per_workgroup;
    int32_t min_rows_per_workgroup;
    int32_t reserved;
    int64_t total_rows;               /* sum of len over all heads                                  */
    int64_t rows_covered;             /* rows of heads whose segments add up to exactly len         */
} hc_plan_info;
hc_status hc_plan_describe(const hc_config* cfg, const hc_head_desc* heads_host, int32_t compute_units,
                           int32_t workgroups_per_cu, hc_plan_info* info, char* err, int32_t err_len);

/* ---- offline stages of Algorithm 1 (host only; no GPU, no context) ------------------------- */
/* Head taxonomy of one layer (Sec. 4.1, Eq. 4-6; App. C.2; Algorithm 1 stage 1) from the calibration results:
 * adjacency [n][n] (uint8, symmetric; non-zero: the two heads' active sets overlap by more than tau_sim)
 * and the stability scores.  Greedy star clustering: the unassigned head with the most unassigned
 * neighbours (lowest index on a tie) becomes a pivot and all its unassigned neighbours its satellites, until
 * no unassigned head has an unassigned neighbour; what is left is an anchor if s_stable >= tau_stable and a
 * volatile head otherwise.  role_out: HC_ROLE_FULL for pivots and volatile heads (both keep their full
 * cache), HC_ROLE_SATELLITE, HC_ROLE_ANCHOR; rep_out: a satellite's pivot, else -1; is_pivot_out (may be
 * NULL): 1 for pivots.  (Sec. 4.1 words it as a split by the similarity score first; App. C.2's procedure is
 * the one implemented.) */
hc_status hc_taxonomy(int32_t n_heads, const uint8_t* adjacency, const double* s_stable, double tau_stable,
                      int32_t* role_out, int32_t* rep_out, int32_t* is_pivot_out);
/* Stability-based budget allocation (Sec. 4.2, Eq. 7-8; Algorithm 1 stage 2): the total (rho N - N_full) L,
 * rho = rho_num / rho_den, is shared among the compressed heads (satellites and anchors) in proportion to
 * 1 / s_stable; full heads get L.  Shares are evaluated in double precision (w = 1.0 / s, sums in head
 * order, share = (total * w) / sum w), rounded down, the slots left over given to the largest fractional
 * parts (lowest index first), so that the budgets add up to the total rounded down; a share above L is cut
 * to L and the rest shared in the same proportion (the paper leaves rounding and that case open).
 * HC_EINVAL if rho N <= N_full (nothing is left for compressed heads). */
hc_status hc_budgets(int32_t n_heads, const int32_t* role, const double* s_stable, int32_t rho_num, int32_t rho_den,
                     int32_t L, int32_t* len_out);

/* ---- hot path ---------------------------------------------------------------------------- */

/* Attention of the decode token over the heterogeneous cache (Algorithm 1, ModelForward over
 * C_GPU; Sec. 4.3): for query head a of sequence b, with h = a / G,
 *     out[b,a,:] = softmax_j( q[b,a,:] . K_{b,h}[j,:] / sqrt(D) ) V_{b,h}[j,:]   over the len
 * resident rows of KV head (b,h); lse[b,a] is the log-sum-exp of those scaled logits.
 *   kv_arena    dev, bf16; rows of 128 elements addressed by the head table's offsets
 *   q           dev, bf16 [B][Hq][D]
 *   out         dev, f32  [B][Hq][D]
 *   lse         dev, f32  [B][Hq]
 *   rep_logits  dev, f32  [num_reps][max_ctx][G], or NULL.  If given, the scaled logits of
 *               every pivot's query group over all ctx positions are stored for the monitor.
 *   stream      hipStream_t (NULL = default stream)
 * bf16 inputs, fp32 accumulation; split over the token axis with a second combine pass. */
hc_status hc_decode_attn(hc_ctx* ctx, const hc_layer* layer, const void* kv_arena, const void* q,
                         float* out, float* lse, float* rep_logits, void* stream);

/* hc_decode_attn for callers that cannot allocate device memory or let a library do it: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same results;
 * the only difference is where the split-K partial results live between the two passes: not in the workspace
 * that hc_layer_create sizes and allocates, but in a fixed array of device memory inside the library (4.3 MB per
 * GPU, there from the moment the library is loaded until the process ends; its address on the context's device
 * is looked up once, in hc_create).  The call allocates and frees nothing, on the host or the device.
 * Limits: the layer's plan may have at most HC_STATIC_MAX_PARTIALS partial results (hc_layer_num_partials;
 * 2 per compute unit plus one per KV head and sequence, i.e. any batch up to 512 head rows on a 256-unit GPU);
 * a larger plan is refused with HC_ESHAPE and nothing is launched.  Every call on one GPU uses the same array,
 * from whatever context: two calls that may overlap (different streams, no ordering between them) race, and the
 * caller must order them; calls on one stream are safe, and nothing needs clearing between calls (the second
 * pass reads only the slots the first pass of the same call wrote). */
hc_status hc_decode_attn_static(hc_ctx* ctx, const hc_layer* layer, const void* kv_arena, const void* q,
                                float* out, float* lse, float* rep_logits, void* stream);

/* Pivot drift monitor (Sec. 4.3, Eq. 9-10; Algorithm 1, the block under "t mod W = 0" with the
 * window read as sliding and tested every step once it holds W values).  For every pivot p:
 *   1. score s[j] = (1/G) sum_g exp(rep_logits[p][j][g] - lse[b, pG+g])        (agg = PROB)
 *      for the candidates j in [sink, ctx-recent); stored to scores (f32 [num_reps][max_ctx]).
 *      With scores_given != 0 this step is skipped and scores is an INPUT.
 *   2. for k = k_mon and every satellite's r: T_k = the k candidates that come first under
 *      (score descending, index ascending); written as ascending lists to topk_idx row of the
 *      pivot (T_{k_mon}) and of each satellite (T_r).  NaN scores rank last; -0 equals +0.
 *   3. inter[p] = |T_{k_mon} ∩ base_idx row p| (entries < 0 in the baseline never match);
 *      pushed into ring[p]; once W values are stored, r_t = [lower-median statistic < tau];
 *      flag[p] = r_t.  On r_t = 1 the baseline row becomes T_{k_mon} and the ring is emptied
 *      (HC_WINDOW_TUMBLING: the ring is emptied after every test).
 * All of topk_idx, base_idx, ring, inter, flag are dev int32 tables as described above;
 * rows of heads that are not pivots (or their satellites, for topk_idx) are left untouched. */
hc_status hc_rep_topk_drift(hc_ctx* ctx, const hc_layer* layer, const float* rep_logits, const float* lse,
                            float* scores, int32_t scores_given,
                            int32_t* topk_idx, int32_t* base_idx, int32_t* ring,
                            int32_t* inter, int32_t* flag, void* stream);

/* AsyncUpdate (Algorithm 1; Sec. 4.3): for every satellite s whose pivot has flag != 0, the r retrieved
 * slots (slots sink+recent .. sink+recent+r-1 of its K and V rows in the arena) are made to hold the
 * host-tier rows of the positions topk_idx[s][0..r-1].  Satellites of pivots with flag == 0 and anchors are
 * not touched (the predicate is evaluated on the device; the call always enqueues).
 *   slot_pos    NULL: slot sink+recent+i <- position topk_idx[s][i] for every i (the whole list crosses
 *               the host link, slots in ascending position order).
 *               Otherwise dev int32 [B*Hkv][max_k], in/out: slot_pos[s][i] is the position that retrieved
 *               slot i of satellite s holds (the caller initialises it with the initial lists).  Only
 *               the difference moves: positions of the list that are not resident go into the slots of
 *               resident positions that left the list, and slot_pos is updated.  Afterwards the resident
 *               set is exactly the list; the slots are no longer in position order, which attention does
 *               not depend on.  Rows that stay are not read again, so the bytes on the host link are
 *               512 * |T_new \ T_old| per satellite.  A slot_pos row that does not hold r distinct
 *               positions is repaired by a full refill.  (The paper replaces the whole satellite cache;
 *               this gives the same resident set.)
 *   host_tier   pinned, bf16; the kernel reads it over the host link
 *   stream      stream to run the gather on (typically a side stream)
 *   wait_event  hipEvent_t or NULL: the stream waits for it first (record it after the monitor)
 *   done_event  hipEvent_t or NULL: recorded after the gather; the attention that next reads this
 *               layer's arena must wait for it (a refill decided at step t is used from t+1). */
hc_status hc_gather_retrieve(hc_ctx* ctx, const hc_layer* layer, const void* host_tier,
                             const int32_t* topk_idx, const int32_t* flag, void* kv_arena,
                             int32_t* slot_pos, void* stream, void* wait_event, void* done_event);

/* Cache update of ModelForward (Algorithm 1: C_GPU is returned updated by ModelForward; Sec. 4.3 keeps the
 * satellites' full K/V on the host): the decode token's rows k_new, v_new (dev bf16 [B][Hkv][D]) become
 * position ctx_b of every head of every sequence b, and ctx_b grows by one.  The paper does not say how a
 * generated token enters compressed heads or the host tier; here:
 *   full heads        row ctx_b of their K and V blocks (which need cap > ctx_b);
 *   compressed heads  the slot of their recent window that held position ctx_b - recent (the window is kept
 *                     as a ring: slot sink + (position - initial ctx) mod recent), so they see the token
 *                     at once; with recent == 0 they do not see it until it is retrieved;
 *   satellites        also row ctx_b of their host-tier block (written by the kernel over the host link),
 *                     so that the position can be retrieved once it has left the window;
 *   pivots            the candidate range [sink, ctx_b - recent) of their top-k grows by the position that
 *                     left the window.
 * Call it before the hc_decode_attn that attends over the token, on the same stream, and after the layer's
 * monitor and gather of the previous step have completed (they read the tables this call updates;
 * hc_decode_step orders it so).  Enqueue-only: every 64 appended tokens the split-K plan is rebalanced on the
 * host and copied to the device in stream order from pinned staging memory that the layer owns; the host does
 * not wait for the stream.  (Not for graph capture: the host's copy of the lengths moves with every call.)
 * Fails with HC_ESHAPE when a head has no room left, before anything is launched. */
hc_status hc_append_kv(hc_ctx* ctx, hc_layer* layer, const void* k_new, const void* v_new, void* kv_arena,
                       void* host_tier, void* stream);
/* Current context length of sequence b of the layer (grows with hc_append_kv); -1 on a bad argument. */
int32_t hc_layer_context(const hc_layer* layer, int32_t b);

/* ---- Prefill-time initialisation (Sec. 4.3, first paragraphs; Algorithm 1, stage 3 before the loop) --------
 * Builds the state decoding starts from, out of the prefill stage's K/V and the last prompt token's
 * queries:
 *   C_GPU: the full heads' K/V rows copied whole; for every compressed head, slots [0, sink) = the first
 *          positions, the next `recent` slots = the last positions, and the other r slots = the r positions
 *          of [sink, ctx - recent) with the head's OWN best scores, in ascending order;
 *   C_CPU: every satellite's whole K/V into its [ctx][2][D] block of host_tier (skipped if NULL);
 *   K_base of every pivot = T_{k_mon} of the pivot's own scores over its satellites' candidate positions;
 *   topk_idx rows of the selecting heads = their lists; slot_pos rows of the satellites (if not NULL) =
 *   their lists; ring rows emptied.
 * Scores: last token's softmax weights over the head's whole context, mean over the query group (or mean of
 * the logits with HC_AGG_LOGIT), then a centred average pooling over positions of odd width `pool` with
 * zero padding and divisor `pool` (App. C.1; 1 = none); decisions in fp32, (score descending, index
 * ascending).
 * kv_prefill: dev bf16; head (b, h)'s K rows [ctx][D] at element offset k_src_off[b*Hkv+h], V rows at
 * v_src_off[..] (HOST arrays of B*Hkv, multiples of 8).  q_last: dev bf16 [B][Hq][D].  work: dev, at least
 * hc_prefill_work_bytes bytes, 256-byte aligned, scratch (hc_prefill_work_layout says where the selecting
 * heads' logits [n][max_ctx][G], scores [n][max_ctx] and the lse [B*Hq] are left, and which table row
 * each selecting head is; head_of needs room for B*Hkv entries).
 * Set-up call: synchronises the stream once (a small table goes to the device), then enqueues.  Must
 * precede any hc_append_kv on the layer. */
size_t hc_prefill_work_bytes(const hc_ctx* ctx, const hc_layer* layer);
hc_status hc_prefill_work_layout(const hc_ctx* ctx, const hc_layer* layer, int32_t* n_selecting, int32_t* head_of,
                                 size_t* logits_off, size_t* scores_off, size_t* lse_off);
hc_status hc_prefill_init(hc_ctx* ctx, hc_layer* layer, const void* kv_prefill, const int64_t* k_src_off,
                          const int64_t* v_src_off, const void* q_last, int32_t pool, void* kv_arena, void* host_tier,
                          int32_t* topk_idx, int32_t* base_idx, int32_t* slot_pos, int32_t* ring, void* work,
                          size_t work_bytes, void* stream);

/* ---- Algorithm 1, the loop over the window's buffered queries at t mod W = 0 (HC_WINDOW_RESCORED) ------
 * Call once per decode step and layer, after hc_decode_attn and BEFORE hc_rep_topk_drift, on the stream
 * of the monitor (hc_decode_step does).  The layer counts the steps of the window: slot = monitored
 * steps since the window was last emptied, 0 when the layer is created (the ring is emptied after every
 * test, so for a ring that started empty slot = steps so far mod W); every call advances it, and
 * hc_layer_set_window_slot sets it for a caller that starts from a ring that is not empty.  The call
 *   - copies the current queries q (dev bf16 [B][Hq][D]) into row `slot` of q_window (dev bf16
 *     [W][B][Hq][D], 16-byte aligned, the caller's: Q_buffer of Algorithm 1);
 *   - at slot == W - 1 (the following hc_rep_topk_drift is the one that tests), for every pivot and every
 *     buffered query k = 0 .. W-2: logits of q_k's group against all of the pivot's K rows as they are now
 *     (a [G (W-1)] x [ctx] x [D] contraction on the matrix cores), their log-sum-exp over the whole
 *     context, the aggregated scores, T_{k_mon} over the current candidate range and |T ∩ K_base|, which
 *     replaces value k of ring[p].  The monitor call then pushes the current step's overlap and decides on
 *     the median of the W re-computed values.  The ring is only touched if it holds exactly W - 1 values.
 * work: device buffer of at least hc_rescore_work_bytes(ctx, layer) bytes, 256-byte aligned, the caller's;
 * contents are scratch (logits, scores and lists of the re-scored queries, laid out as
 * hc_rescore_work_layout reports: place i holds the last query k with k mod items_per_pass == i, which
 * is what the tests read).  Uses the context's selection workspaces like a batched monitor call:
 * stream-order it with other monitor calls.
 * Enqueue-only, no allocation.  W == 1 or a layer without pivots: only the copy happens.  Which row the
 * queries go to and whether the passes run is decided on the host when the call is made, so a captured
 * graph of this call would repeat one step of the window: capture whole windows (W calls) or none. */
size_t hc_rescore_work_bytes(const hc_ctx* ctx, const hc_layer* layer);
/* Byte offsets of the passes' results inside `work` and how many queries a pass holds
 * (min(8, 32 / G)): logits [items][num_reps][max_ctx][G] f32, scores [items][num_reps][max_ctx] f32,
 * lse [items][B*Hq] f32, lists [items][B*Hkv][max_k] int32.  Any pointer may be NULL. */
hc_status hc_rescore_work_layout(const hc_ctx* ctx, const hc_layer* layer, int32_t* items_per_pass, size_t* logits_off,
                                 size_t* scores_off, size_t* lse_off, size_t* topk_off);
hc_status hc_rescore_window(hc_ctx* ctx, hc_layer* layer, const void* kv_arena, const void* q, void* q_window,
                            const int32_t* base_idx, int32_t* ring, void* work, size_t work_bytes, void* stream);
/* The layer's count of steps inside the current window (-1: bad layer), and its setter (0 .. W-1). */
int32_t hc_layer_window_slot(const hc_layer* layer);
hc_status hc_layer_set_window_slot(hc_layer* layer, int32_t slot);

/* One decode step over a stack of layers (Algorithm 1, the body of the loop over t, for every layer):
 * for each layer in order, hc_decode_attn on main_stream, then hc_rep_topk_drift and hc_gather_retrieve
 * on side_stream (NULL = on main_stream, no overlap; a stack of at most layers_per_group layers is handled that way
 * too, since a single group's side work has nothing to overlap).  Layers are handled in groups of layers_per_group
 * (1..HC_MAX_GROUP; 8 measured best at 32 layers of 224K): the group's appended tokens (k_new / v_new) in
 * one launch, the group's attentions, then one cross-stream event, then ONE batched monitor and ONE
 * batched gather for the whole group, which overlap the attention of the following groups; with
 * HC_WINDOW_RESCORED also one launch that buffers the group's queries (on main_stream: q may be
 * overwritten as soon as the call returns) and, at the window's last step, the re-scoring passes of the
 * whole group ahead of its monitor.  The attention of a layer at the next call waits for that layer's side work of this call, so
 * a refill decided at step t is used from step t+1.  Launching from native code keeps the host ahead
 * of the GPU.  All buffers are the caller's, as in the three calls; scores == NULL (or a layer without
 * pivots) skips monitor and gather for that layer; host_tier == NULL skips the gather.  Layers whose
 * monitors overlap other layers' attention need their own rep_logits, scores, lse, out.  The context
 * holds one selection workspace per position in a group; hc_rep_topk_drift uses the first, so a direct
 * call must be stream-ordered with this call's side work.  Every layer's arguments are checked before the first
 * launch, so a refused call leaves every layer as it was.  Enqueue-only; not meant for graph capture
 * (it uses per-layer events). */
typedef struct {
    hc_layer* layer;
    const void* kv_arena;     /* dev; also written by the gather */
    const void* host_tier;    /* pinned, or NULL */
    const void* q;            /* dev bf16 [B][Hq][D] */
    float* out;               /* dev [B][Hq][D] */
    float* lse;               /* dev [B][Hq] */
    float* rep_logits;        /* dev [num_reps][max_ctx][G] */
    float* scores;            /* dev [num_reps][max_ctx], or NULL */
    int32_t* topk_idx;
    int32_t* base_idx;
    int32_t* ring;
    int32_t* inter;
    int32_t* flag;
    int32_t* slot_pos;        /* dev [B*Hkv][max_k] in/out, or NULL: see hc_gather_retrieve */
    const void* k_new;        /* dev bf16 [B][Hkv][D]: with v_new, the token to append before attention  */
    const void* v_new;        /*   (hc_append_kv); both NULL: the context does not grow                  */
    void* q_window;           /* HC_WINDOW_RESCORED: dev bf16 [W][B][Hq][D] and the work buffer of               */
    void* rescore_work;       /*   hc_rescore_window;                                                            */
    size_t rescore_work_bytes;/*   ignored in the other window modes                                              */
} hc_layer_io;
hc_status hc_decode_step(hc_ctx* ctx, const hc_layer_io* layers, int32_t n_layers, int32_t layers_per_group,
                         void* main_stream, void* side_stream);

#ifdef __cplusplus
}
#endif
#endif
