// hc_internal.h -- shared declarations of the HIP library (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <utility>
#include <mutex>
#include <unordered_map>
#include <vector>

#include "../../include/hc.h"

constexpr int HC_D = 128;            // head dimension the kernels are written for
constexpr int HC_UNIT_ROWS = 32;     // split-K granule: 4 waves x 8 rows
constexpr int HC_SEL_CHUNK = 1024;   // candidates per workgroup in the selection passes
constexpr int HC_RADIX_BINS = 2048;  // 11-bit digits (11 + 11 + 10 bits of the 32-bit key)

// One KV head as the kernels see it.
struct HeadDev {
    int64_t k_off, v_off, tier_off;
    int32_t len, ctx;      // ctx (and len of a full head) grow on the device with every appended token
    int32_t rep_slot;      // >= 0: this full head is a pivot and owns that slot of rep_logits
    int32_t part_begin;    // first split-K partial of this head
    int32_t part_count;
    int32_t role;          // HC_ROLE_*
    int32_t sink, recent;  // compressed heads
    int32_t ctx0;          // context length when the layer was created: anchors the ring of recent slots
    int32_t tail_seg;      // full head: the segment that holds its last row, and the workgroup whose
    int32_t tail_blk;      //   descriptor carries a copy of that segment (-1: none does)
    int32_t pad;
};

// A contiguous run of rows of one head handled by one workgroup of the split pass; self-contained so
// that a workgroup can start streaming after a single descriptor read.
struct SegDev {
    int64_t k_off, v_off;          // element offsets of the head's K and V blocks in the arena
    int32_t bh, row_begin, row_end, slot;
    int32_t rep_slot;
    int32_t pad;
};

// What workgroup b of the split pass does: its first segment inline, any further ones (when its
// share of rows crosses a head boundary) in segs[extra_begin, extra_end).
struct BlkDev {
    SegDev first;
    int32_t extra_begin, extra_end, pad0, pad1;
};
static_assert(sizeof(SegDev) == 40 && sizeof(BlkDev) == 56, "descriptor layout");

// One pivot of the layer.
struct RepDev {
    int32_t bh;                       // table row b*Hkv+h
    int32_t lo, hi;                   // candidate positions [lo, hi)
    int32_t nk;                       // distinct set sizes
    int32_t k[HC_MAX_K_PER_REP];      // k[0] = k_mon
    int32_t nchunk;                   // ceil((hi-lo)/HC_SEL_CHUNK)
    int32_t out_begin, out_count;     // this pivot's lists: outs[out_begin, out_begin + out_count)
};

// One index list to emit: row `row` of topk_idx gets T_k with k = rep.k[kslot].
struct OutDev {
    int32_t rep, kslot, row, is_mon;
};

// State of one pivot's logit filter: written by the monitor's decision kernel, read by the next step's split pass.
// A row of the pivot is kept for the monitor if sum_g 2^(t_g - ref[g]) >= cutsum (t: scaled logit in log2 units).
struct RepFilter {
    float cutsum;          // 0: every candidate row is kept
    float ref[8];          // the log-sum-exp of each query head of the group at the step that set the filter, log2 units
    int32_t armed;         // 0 until a decision has set the filter
    int32_t pad[6];
};
static_assert(sizeof(RepFilter) == 64, "filter state layout");

// Where a head's K and V rows of the prefill stage are (element offsets in the caller's prefill buffer).
struct PreSrc {
    int64_t k_off, v_off;
};

// One satellite to refill.
struct SatDev {
    int32_t bh, rep_bh, r, first_slot;   // first_slot = sink + recent
};

struct hc_monitor_ws {
    uint32_t* hist = nullptr;      // [max_reps][HC_MAX_K_PER_REP][3][HC_RADIX_BINS]
    uint32_t* sel = nullptr;       // [max_reps][HC_MAX_K_PER_REP][4]: prefix, remaining k, (tau, need)
    uint32_t* misc = nullptr;      // [max_reps][4]: spare
    uint32_t* cnt = nullptr;       // [max_reps][HC_MAX_K_PER_REP][max_chunks][2]: greater, equal
    uint32_t* bitmap = nullptr;    // [max_reps][max_ctx/32]
    uint32_t* hits = nullptr;      // [max_reps][max_chunks+1]: per-chunk |T ∩ baseline|
    bool dirty = true;             // histograms / bitmap not known to be clear (first call, or a call that failed midway)
};

struct hc_ctx {
    uint32_t magic;
    hc_config cfg;
    int G;
    int n_cu;
    int wg_per_cu;
    unsigned long long* tune_stamps = nullptr;   // non-null only inside hc_layer_tune: per-workgroup start / rows-done times
    float share_weights[16];     // by die and dispatch slot, see hc_set_share_weights
    int gather_workgroups = 96, gather_threads = 256;   // launch shape of the gather (hc_set_gather_shape)
    float filter_margin = 0.f;   // > 0: pivot logits are filtered (hc_set_logit_filter); layers created afterwards carry the buffers
    int filter_min_candidates = 0;   // ... if one of their pivots has at least this many candidate positions
    int side_lds_total = 81 * 1024;   // > 0: LDS bytes every side-stream workgroup of hc_decode_step reserves (hc_set_side_lds)
    bool side_pad_now = false;   // set while hc_decode_step enqueues a group's side work on a stream of its own
    int device;
    char err[512];
    std::vector<std::pair<hipEvent_t, hipEvent_t>> timing;   // optional timing hook: one pair per split-pass launch
    size_t timing_next = 0;
    // split-K partial workspace
    float* part_acc = nullptr;   // [slots][G][D]
    float* part_ml = nullptr;    // [slots][G][2]  (running max in log2 units, sum)
    size_t part_slots = 0;
    float* static_scratch = nullptr;   // this device's address of the fixed scratch array of hc_decode_attn_static
    // selection workspace, sized for max_reps pivots; one copy per layer of a batched monitor call
    int max_reps = 0;
    uint32_t* ws_base = nullptr;   // the one allocation behind all lanes
    hc_monitor_ws ws[HC_MAX_GROUP];
    int max_chunks = 0;
    int monitor_span = 0;          // chunks per workgroup of the selection passes; 0: chosen per launch
    // gather workspace, one copy per layer of a batched call: the (slot, position) pairs of a refill
    int32_t* pair_slot = nullptr;  // [HC_MAX_GROUP][B*Hkv][max_k]
    int32_t* pair_pos = nullptr;   // [HC_MAX_GROUP][B*Hkv][max_k]
    int32_t* npairs = nullptr;     // [HC_MAX_GROUP][B*Hkv]
};

struct hc_layer {
    uint32_t magic;
    hc_ctx* ctx;
    int n_heads;
    int n_blocks, n_partials, n_segs;
    int n_reps, n_outs, n_sats;
    int max_r;                     // largest r among satellites
    int max_nchunk;
    int max_nk;                    // largest number of distinct set sizes of a pivot
    int max_k_any = 1;             // largest set size of any pivot
    std::vector<int32_t> rep_slot_of;   // [B*Hkv]
    std::vector<hc_head_desc> hd_host;  // the head table as it is now (lengths grow with appended tokens)
    std::vector<int32_t> ctx0_host;     // [B*Hkv] context lengths at creation
    std::vector<int32_t> rep_lo_host, rep_recent_host;   // per pivot: first candidate, recent slots of its satellites
    int appended_since_plan = 0;
    long long total_appended = 0;       // tokens appended since creation
    // prefill-time initialisation: the heads that select (compressed heads by their own scores, pivots for their
    // baseline sets), one list each
    int n_sel = 0, sel_max_nchunk = 1, sel_max_len = 1;
    int prefill_unfit_head = -1;        // a compressed head whose slots the selection cannot fill (list longer than max_k)
    RepDev* sel_reps = nullptr;
    OutDev* sel_outs = nullptr;
    PreSrc* pre_src = nullptr;          // [n_heads]
    int32_t* rep_slot_dev = nullptr;    // [n_heads]: device copy of rep_slot_of
    std::vector<int32_t> sel_head_host; // table rows of the selecting heads, in the order of sel_reps
    int window_slot = 0;                // hc_decode_step with a re-scored window: monitored steps since the window was emptied
    // A rebalanced plan goes to the device from pinned staging memory the layer owns, so that the copy is
    // asynchronous and the host need not wait for it: two staging buffers alternate, each guarded by an event
    // recorded behind its copy (waited for only if that buffer comes round again before its copy has run).
    char* plan_stage[2] = {nullptr, nullptr};
    size_t plan_stage_bytes = 0;
    hipEvent_t plan_copied[2] = {nullptr, nullptr};
    int plan_next = 0;
    int seg_capacity = 0;               // device room in segs (a rebalanced plan may have a few more segments)
    int blk_capacity = 0;               // device room in blks (a short layer gets more workgroups as it grows)
    HeadDev* heads = nullptr;
    SegDev* segs = nullptr;
    BlkDev* blks = nullptr;        // [n_blocks]
    RepDev* reps = nullptr;
    OutDev* outs = nullptr;
    SatDev* sats = nullptr;
    // pivot-logit filter (only for layers created while the context's filter is on; all device memory)
    RepFilter* filt = nullptr;     // [n_reps]
    int32_t* surv_pos = nullptr;   // [n_reps][max_ctx] positions of the rows the split pass kept, by segment
    int32_t* dense_pos = nullptr;  // [n_reps][max_ctx] the same positions, all of a pivot's in one ascending run
    int32_t* seg_cnt = nullptr;    // [seg_capacity] rows kept per pivot segment
    RepDev* vreps = nullptr;       // [n_reps] the pivots as the selection passes see them over the kept rows (lo = 0, hi = rows kept)
    int32_t* need = nullptr;       // [n_reps] != 0: the check of this step's filter failed, the dense passes take over
    uint16_t* q_keep = nullptr;    // [n_reps][G][D] the pivots' queries of the last attention call
    uint32_t* mon_counts = nullptr;// [n_reps][4] tests, triggers, steps decided by the dense fallback, rows kept at the last step
    const void* last_arena = nullptr;   // the arena of the last attention call with pivot logits (the fallback reads K from it)
    bool filter_armed = false;     // a monitor call has set the filter: the selection passes are launched for few rows
    hipEvent_t ev_attn = nullptr;  // hc_decode_step: this layer's attention has been enqueued / its side work is done
    hipEvent_t ev_side = nullptr;
    hipEvent_t pending_ev = nullptr;   // side work of the previous hc_decode_step that this layer's attention must wait for
};

constexpr uint32_t HC_CTX_MAGIC = 0x48435458u;    // "HCTX"
constexpr uint32_t HC_LAYER_MAGIC = 0x48434c59u;  // "HCLY"

hc_status hc_fail(hc_ctx* ctx, hc_status st, const char* fmt, ...);
// Does this layer's split pass filter the pivot logits (and its monitor read them that way)?
inline bool hc_layer_filtered(const hc_ctx* ctx, const hc_layer* L)
{
    return ctx->filter_margin > 0.f && L->filt != nullptr && ctx->cfg.agg == HC_AGG_PROB;
}
hc_status hc_hip_fail(hc_ctx* ctx, hipError_t e, const char* what);

#define HC_HIP(ctx, call)                                             \
    do {                                                              \
        hipError_t e_ = (call);                                       \
        if (e_ != hipSuccess) return hc_hip_fail((ctx), e_, #call);   \
    } while (0)

// kernel launchers (one translation unit each).  Monitor and gather take a batch of 1..HC_MAX_GROUP
// layers and handle it with the launches of one layer.
struct hc_monitor_call {
    const hc_layer* L;
    const float* rep_logits;
    const float* lse;
    float* scores;
    int32_t *topk_idx, *base_idx, *ring, *inter, *flag;
    int store_slot = -1;   // >= 0: a re-scored query of the window: only its overlap is kept, as value store_slot of the
                           // ring (if the ring is one short of full), and baseline, inter, flag are left alone;
                           // -2: lists only (prefill-time selection): no overlap, no decision, tables untouched
    // prefill-time selection runs over its own list of heads instead of the layer's pivots
    const RepDev* reps = nullptr;
    const OutDev* outs = nullptr;
    int n_reps = 0, n_outs = 0, max_nchunk = 0, max_nk = 0;
    const void* arena = nullptr;   // the layer's K/V arena, for a layer that filters its pivot logits (nullptr: the one
                                   // its last attention call was given)
};
struct hc_gather_call {
    const hc_layer* L;
    const void* tier;
    const int32_t* topk_idx;
    const int32_t* flag;
    void* arena;
    int32_t* slot_pos;     // or nullptr
};
hc_status hc_launch_attn(hc_ctx* ctx, const hc_layer* L, const void* arena, const void* q, float* out,
                         float* lse, float* rep_logits, hipStream_t st);
hc_status hc_launch_attn_static(hc_ctx* ctx, const hc_layer* L, const void* arena, const void* q, float* out,
                                float* lse, float* rep_logits, hipStream_t st);
hc_status hc_attn_static_scratch(hc_ctx* ctx, float** base);     // at context creation, with the context's device current
hc_status hc_launch_rep_logits(hc_ctx* ctx, int n, const hc_layer* const* layers, const void* const* arenas,
                               float* const* rep_logits, hipStream_t st);
hc_status hc_launch_monitor(hc_ctx* ctx, int n, const hc_monitor_call* calls, int scores_given, hipStream_t st);
hc_status hc_launch_gather(hc_ctx* ctx, int n, const hc_gather_call* calls, hipStream_t st);
hc_status hc_gather_set_lds_limit();     // once per process, at context creation
hc_status hc_monitor_set_lds_limit();
hc_status hc_attn_set_lds_limit();
// Dynamic LDS for a launch of side-stream kernel fn that itself needs dyn_needed bytes.  Beside the attention pass
// (side_pad_now) the workgroup's LDS is brought up to side_lds_total bytes, more than half of a compute unit's: a
// compute unit then never holds more than one workgroup of the side stream, whatever got there first, and always has
// room (LDS, registers, wave slots) for its two workgroups of the attention pass.
inline unsigned hc_side_lds(const hc_ctx* ctx, const void* fn, unsigned dyn_needed)
{
    if (!ctx->side_pad_now || ctx->side_lds_total <= 0) return dyn_needed;
    static std::unordered_map<const void*, unsigned> static_lds;      // of the kernels seen so far (a property of the code)
    static std::mutex guard;
    std::lock_guard<std::mutex> lock(guard);
    auto it = static_lds.find(fn);
    if (it == static_lds.end()) {
        hipFuncAttributes a{};
        if (hipFuncGetAttributes(&a, fn) != hipSuccess) return dyn_needed;
        it = static_lds.emplace(fn, (unsigned)a.sharedSizeBytes).first;
    }
    const unsigned st = it->second;
    const unsigned want = (unsigned)ctx->side_lds_total > st ? (unsigned)ctx->side_lds_total - st : 0u;
    return want > dyn_needed ? want : dyn_needed;
}
constexpr int HC_LDS_PER_CU = 160 * 1024;
inline hipError_t hc_allow_lds(const void* fn)       // lets fn be launched with any dynamic LDS a compute unit can give
{
    hipFuncAttributes a{};
    hipError_t e = hipFuncGetAttributes(&a, fn);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, HC_LDS_PER_CU - (int)a.sharedSizeBytes);
}    // likewise
// Work buffer of the window re-scoring pass (offsets in bytes, item sizes in elements).
constexpr int HC_RESCORE_MAX_BLOCKS = 512;
struct hc_rescore_layout {
    size_t logits_off, scores_off, lse_off, topk_off, part_off, scratch_off, bytes;
    size_t logits_item, scores_item, lse_item, topk_item;
};
int hc_rescore_items_per_pass(const hc_ctx* ctx);
hc_rescore_layout hc_rescore_plan(const hc_ctx* ctx, const hc_layer* L);
hc_status hc_launch_rescore_push(hc_ctx* ctx, int n, const void* const* q, void* const* dst, hipStream_t st);
struct hc_logits_job {
    const hc_layer* L;
    const RepDev* reps;        // the heads to score against, n_heads of them; max_len: the longest
    int n_heads, max_len;
    const void* arena;         // where their K rows are (see src)
    const PreSrc* src;
    const void* q;             // first query
    float* logits;
    size_t logits_item;
    float* lse;
    size_t lse_item;
    float* part;
};
hc_status hc_launch_logits_lse(hc_ctx* ctx, int n_jobs, const hc_logits_job* jobs, int n_items, hipStream_t st);
hc_logits_job hc_rescore_job(const hc_ctx* ctx, const hc_layer* L, const void* arena, const void* q_window, int first, void* work);
// prefill-time initialisation
constexpr int HC_MAX_POOL = 63;
struct hc_prefill_layout {
    size_t logits_off, scores_off, lse_off, part_off, scratch_off, bytes;
};
hc_prefill_layout hc_prefill_plan(const hc_ctx* ctx, const hc_layer* L);
hc_status hc_launch_prefill_scores(hc_ctx* ctx, const hc_layer* L, const float* logits, const float* lse, float* scores, int pool,
                                   hipStream_t st);
hc_status hc_launch_prefill_place(hc_ctx* ctx, const hc_layer* L, const void* kv_prefill, void* arena, void* tier,
                                  const int32_t* topk_idx, int32_t* base_idx, int32_t* slot_pos, int32_t* ring, hipStream_t st);
struct hc_append_call {
    const hc_layer* L;
    const void* k_new;
    const void* v_new;
    void* arena;
    void* tier;            // or nullptr (a layer without satellites)
};
hc_status hc_launch_append(hc_ctx* ctx, int n, const hc_append_call* calls, hipStream_t st);
