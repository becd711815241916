// hc_host.hip -- life cycle, validation and work planning of the HeteroCache decode library.
//
// Everything here runs on the host at set-up time.  The per-step entry points at the bottom only
// validate their arguments and enqueue kernels (hc_attn.hip, hc_monitor.hip, hc_gather.hip).
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <limits.h>

#include <algorithm>
#include <new>
#include <utility>

#include "hc_internal.h"

// Relative share of rows of a split-pass workgroup by die (workgroup index mod 8) and dispatch slot
// (first / second half of the indices): [die * 2 + slot].  Measured on MI355X with equal shares at the
// 224K-context shape (about 940 rows per workgroup), in back-to-back launches: the second workgroup on
// a compute unit finishes about 2 us (6 %) after the first, and workgroups on odd dies about 2.5 us (7 %)
// after those on even dies.  These weights equalise the mean finish time of the 16 classes there (the pass
// ends about 1.5 us earlier); they are applied only to passes long enough for such corrections to matter.
static const float DEFAULT_SHARE_WEIGHTS[16] = {1.07f, 0.99f, 1.02f, 0.95f, 1.06f, 0.99f, 0.99f, 0.92f,
                                                1.06f, 0.99f, 0.99f, 0.92f, 1.08f, 1.01f, 1.02f, 0.95f};

hc_status hc_fail(hc_ctx* ctx, hc_status st, const char* fmt, ...)
{
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof ctx->err, fmt, ap);
        va_end(ap);
    }
    return st;
}

hc_status hc_hip_fail(hc_ctx* ctx, hipError_t e, const char* what)
{
    return hc_fail(ctx, e == hipErrorOutOfMemory ? HC_ENOMEM : HC_EHIP, "%s: %s", what, hipGetErrorString(e));
}

extern "C" const char* hc_strerror(hc_status st)
{
    switch (st) {
    case HC_OK: return "ok";
    case HC_EINVAL: return "invalid argument";
    case HC_ESHAPE: return "unsupported shape";
    case HC_ENOMEM: return "out of memory";
    case HC_EHIP: return "HIP call failed";
    case HC_ESTATE: return "object in wrong state";
    }
    return "unknown status";
}

extern "C" const char* hc_last_error(const hc_ctx* ctx)
{
    return (ctx && ctx->magic == HC_CTX_MAGIC) ? ctx->err : "invalid context";
}

static bool ctx_ok(const hc_ctx* c) { return c && c->magic == HC_CTX_MAGIC; }
static bool layer_ok(const hc_layer* l) { return l && l->magic == HC_LAYER_MAGIC && ctx_ok(l->ctx); }

// Words of selection workspace per pivot that a monitor call clears before use:
// digit histograms (one shared first pass, then one per set size for passes two and three),
// the selection state and the intersection accumulator / ticket.
static size_t rep_hist_words() { return (size_t)(1 + 2 * HC_MAX_K_PER_REP) * HC_RADIX_BINS; }

static hc_status check_config(const hc_config* cfg)
{
    if (!cfg) return HC_EINVAL;
    if (cfg->D != HC_D) return HC_ESHAPE;
    if (cfg->B < 1 || cfg->Hkv < 1 || cfg->Hq < 1 || cfg->Hq % cfg->Hkv != 0) return HC_EINVAL;
    const int G = cfg->Hq / cfg->Hkv;
    if (G != 1 && G != 2 && G != 4 && G != 8) return HC_ESHAPE;
    if (cfg->max_ctx < 64 || cfg->max_ctx % 64 != 0 || cfg->max_ctx > (1 << 24)) return HC_ESHAPE;
    if (cfg->max_k < 1 || cfg->max_k > cfg->max_ctx) return HC_EINVAL;
    if (cfg->window < 1 || cfg->window > HC_MAX_WINDOW) return HC_EINVAL;
    if (cfg->metric != HC_METRIC_OVERLAP && cfg->metric != HC_METRIC_JACCARD) return HC_EINVAL;
    if (cfg->agg != HC_AGG_PROB && cfg->agg != HC_AGG_LOGIT) return HC_EINVAL;
    if (cfg->window_mode < HC_WINDOW_SLIDING || cfg->window_mode > HC_WINDOW_RESCORED) return HC_EINVAL;
    if (cfg->tau_den < 1 || cfg->tau_num < 0) return HC_EINVAL;
    if ((int64_t)cfg->B * cfg->Hkv > (1 << 20)) return HC_ESHAPE;
    return HC_OK;
}

extern "C" hc_status hc_create(const hc_config* cfg, hc_ctx** out)
{
    if (!cfg || !out) return HC_EINVAL;
    *out = nullptr;
    const hc_status cs = check_config(cfg);
    if (cs != HC_OK) return cs;
    const int G = cfg->Hq / cfg->Hkv;

    hc_ctx* c = new (std::nothrow) hc_ctx();
    if (!c) return HC_ENOMEM;
    c->magic = HC_CTX_MAGIC;
    c->cfg = *cfg;
    c->G = G;
    c->wg_per_cu = 2;
    for (int i = 0; i < 16; ++i) c->share_weights[i] = DEFAULT_SHARE_WEIGHTS[i];
    c->err[0] = 0;
    hipDeviceProp_t prop;
    hipError_t e = hipGetDevice(&c->device);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, c->device);
    if (e != hipSuccess) {
        delete c;
        return HC_EHIP;
    }
    c->n_cu = prop.multiProcessorCount;

    // pivots are at most half of the heads; the prefill-time selection runs over up to all of them
    c->max_reps = std::max(1, cfg->B * cfg->Hkv);
    c->max_chunks = (cfg->max_ctx + HC_SEL_CHUNK - 1) / HC_SEL_CHUNK;
    const size_t hist_w = (size_t)c->max_reps * rep_hist_words();
    const size_t sel_w = (size_t)c->max_reps * HC_MAX_K_PER_REP * 4;
    const size_t misc_w = (size_t)c->max_reps * 4;
    const size_t cnt_w = (size_t)c->max_reps * HC_MAX_K_PER_REP * c->max_chunks * 2;
    const size_t bm_w = (size_t)c->max_reps * (cfg->max_ctx / 32);
    const size_t hits_w = (size_t)c->max_reps * (c->max_chunks + 1);
    const size_t lane_w = hist_w + sel_w + misc_w + cnt_w + bm_w + hits_w;
    uint32_t* base = nullptr;
    e = hipMalloc((void**)&base, HC_MAX_GROUP * lane_w * sizeof(uint32_t));
    if (e != hipSuccess) {
        delete c;
        return e == hipErrorOutOfMemory ? HC_ENOMEM : HC_EHIP;
    }
    c->ws_base = base;
    {
        const size_t rows = (size_t)cfg->B * cfg->Hkv;
        const size_t pair_w = (size_t)HC_MAX_GROUP * rows * cfg->max_k;
        int32_t* g = nullptr;
        e = hipMalloc((void**)&g, (2 * pair_w + (size_t)HC_MAX_GROUP * rows) * sizeof(int32_t));
        if (e != hipSuccess) {
            (void)hipFree(base);
            delete c;
            return e == hipErrorOutOfMemory ? HC_ENOMEM : HC_EHIP;
        }
        c->pair_slot = g;
        c->pair_pos = g + pair_w;
        c->npairs = g + 2 * pair_w;
        (void)hc_gather_set_lds_limit();
        (void)hc_monitor_set_lds_limit();
        (void)hc_attn_set_lds_limit();
        // the fixed scratch of hc_decode_attn_static: its address on this device (left null if the lookup fails;
        // that entry point then refuses to run, the others do not need it)
        if (hc_attn_static_scratch(c, &c->static_scratch) != HC_OK) c->static_scratch = nullptr;
    }
    for (int i = 0; i < HC_MAX_GROUP; ++i) {
        hc_monitor_ws& w = c->ws[i];
        w.hist = base + (size_t)i * lane_w;
        w.sel = w.hist + hist_w;
        w.misc = w.sel + sel_w;
        w.cnt = w.misc + misc_w;
        w.bitmap = w.cnt + cnt_w;
        w.hits = w.bitmap + bm_w;
        w.dirty = true;
    }
    *out = c;
    return HC_OK;
}

extern "C" hc_status hc_destroy(hc_ctx* ctx)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    (void)hipFree(ctx->ws_base);
    (void)hipFree(ctx->pair_slot);
    (void)hipFree(ctx->part_acc);
    (void)hipFree(ctx->part_ml);
    ctx->magic = 0;
    delete ctx;
    return HC_OK;
}

extern "C" hc_status hc_set_split(hc_ctx* ctx, int32_t workgroups_per_cu, int32_t compute_units)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    if (workgroups_per_cu < 1 || workgroups_per_cu > 16 || compute_units < 0 || compute_units > 4096)
        return hc_fail(ctx, HC_EINVAL, "hc_set_split: workgroups_per_cu 1..16, compute_units 0..4096");
    ctx->wg_per_cu = workgroups_per_cu;
    if (compute_units > 0) ctx->n_cu = compute_units;
    return HC_OK;
}

extern "C" hc_status hc_get_share_weights(const hc_ctx* ctx, float* weights16)
{
    if (!ctx_ok(ctx) || !weights16) return HC_ESTATE;
    for (int i = 0; i < 16; ++i) weights16[i] = ctx->share_weights[i];
    return HC_OK;
}

extern "C" hc_status hc_set_share_weights(hc_ctx* ctx, const float* weights16)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    for (int i = 0; i < 16; ++i) {
        const float w = weights16 ? weights16[i] : DEFAULT_SHARE_WEIGHTS[i];
        if (!(w >= 0.25f && w <= 4.0f)) return hc_fail(ctx, HC_EINVAL, "hc_set_share_weights: weight %d outside 0.25..4", i);
        ctx->share_weights[i] = w;
    }
    return HC_OK;
}

extern "C" hc_status hc_set_logit_filter(hc_ctx* ctx, float margin, int32_t min_candidates)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    if (!(margin == 0.f || (margin >= 1.f && margin <= 1.0e6f)) || min_candidates < 0)
        return hc_fail(ctx, HC_EINVAL, "hc_set_logit_filter: margin 0 (off) or 1 .. 1e6, min_candidates >= 0");
    ctx->filter_margin = margin;
    ctx->filter_min_candidates = min_candidates;
    return HC_OK;
}

extern "C" hc_status hc_set_side_lds(hc_ctx* ctx, int32_t bytes)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    if (bytes != 0 && (bytes <= HC_LDS_PER_CU / 2 || bytes > 100 * 1024))
        return hc_fail(ctx, HC_EINVAL, "hc_set_side_lds: 0, or more than half of a compute unit's LDS (%d bytes) up to 100 KB", HC_LDS_PER_CU / 2);
    ctx->side_lds_total = bytes;
    return HC_OK;
}

extern "C" hc_status hc_set_gather_shape(hc_ctx* ctx, int32_t workgroups, int32_t threads)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    if (workgroups < 1 || workgroups > 4096 || (threads != 64 && threads != 128 && threads != 256))
        return hc_fail(ctx, HC_EINVAL, "hc_set_gather_shape: 1..4096 workgroups of 64, 128 or 256 threads");
    ctx->gather_workgroups = workgroups;
    ctx->gather_threads = threads;
    return HC_OK;
}

extern "C" hc_status hc_set_monitor_span(hc_ctx* ctx, int32_t span)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    if (span < 0 || span > 64) return hc_fail(ctx, HC_EINVAL, "hc_set_monitor_span: 0 (automatic) or 1..64");
    ctx->monitor_span = span;
    return HC_OK;
}

extern "C" hc_status hc_set_timing_events(hc_ctx* ctx, void* const* ev_begin, void* const* ev_end, int32_t n)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    if (n < 0 || (n > 0 && (ev_begin == nullptr || ev_end == nullptr)))
        return hc_fail(ctx, HC_EINVAL, "hc_set_timing_events: n >= 0 and two arrays of n events");
    for (int i = 0; i < n; ++i)
        if (ev_begin[i] == nullptr || ev_end[i] == nullptr)
            return hc_fail(ctx, HC_EINVAL, "hc_set_timing_events: pair %d has a NULL event", i);
    ctx->timing.clear();
    ctx->timing_next = 0;
    for (int i = 0; i < n; ++i) ctx->timing.emplace_back((hipEvent_t)ev_begin[i], (hipEvent_t)ev_end[i]);
    return HC_OK;
}

static hc_status ensure_partials(hc_ctx* ctx, size_t slots)
{
    if (slots <= ctx->part_slots) return HC_OK;
    HC_HIP(ctx, hipDeviceSynchronize());      // set-up time: nothing may still read the old buffers
    (void)hipFree(ctx->part_acc);
    (void)hipFree(ctx->part_ml);
    ctx->part_acc = ctx->part_ml = nullptr;
    ctx->part_slots = 0;
    HC_HIP(ctx, hipMalloc((void**)&ctx->part_acc, slots * ctx->G * HC_D * sizeof(float)));
    HC_HIP(ctx, hipMalloc((void**)&ctx->part_ml, slots * ctx->G * 2 * sizeof(float)));
    ctx->part_slots = slots;
    return HC_OK;
}

template <class T>
static hc_status upload(hc_ctx* ctx, const std::vector<T>& v, T** dev, size_t capacity = 0)
{
    *dev = nullptr;
    const size_t n = std::max<size_t>(std::max<size_t>(1, v.size()), capacity);
    HC_HIP(ctx, hipMalloc((void**)dev, n * sizeof(T)));
    if (!v.empty()) HC_HIP(ctx, hipMemcpy(*dev, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice));
    return HC_OK;
}

static void layer_free(hc_layer* L)
{
    (void)hipFree(L->heads);
    (void)hipFree(L->segs);
    (void)hipFree(L->blks);
    (void)hipFree(L->reps);
    (void)hipFree(L->outs);
    (void)hipFree(L->sats);
    (void)hipFree(L->sel_reps);
    (void)hipFree(L->sel_outs);
    (void)hipFree(L->pre_src);
    (void)hipFree(L->rep_slot_dev);
    (void)hipFree(L->filt);
    (void)hipFree(L->surv_pos);
    (void)hipFree(L->dense_pos);
    (void)hipFree(L->seg_cnt);
    (void)hipFree(L->vreps);
    (void)hipFree(L->need);
    (void)hipFree(L->q_keep);
    (void)hipFree(L->mon_counts);
    if (L->ev_attn) (void)hipEventDestroy(L->ev_attn);
    if (L->ev_side) (void)hipEventDestroy(L->ev_side);
    for (int i = 0; i < 2; ++i) {
        if (L->plan_stage[i]) (void)hipHostFree(L->plan_stage[i]);
        if (L->plan_copied[i]) (void)hipEventDestroy(L->plan_copied[i]);
    }
    L->magic = 0;
    delete L;
}

// Everything hc_layer_create derives from the head table, on the host only.
struct Plan {
    std::vector<HeadDev> heads;
    std::vector<SegDev> segs;
    std::vector<int32_t> blk_seg;
    std::vector<BlkDev> blks;
    std::vector<RepDev> reps;
    std::vector<OutDev> outs;
    std::vector<SatDev> sats;
    std::vector<int32_t> rep_slot_of;
    int n_blocks = 0, max_r = 0, max_nchunk = 1;
    int64_t total_rows = 0;
};

struct ErrBuf {
    char* buf;
    size_t len;
    hc_status fail(hc_status st, const char* fmt, ...) const
    {
        if (buf && len) {
            va_list ap;
            va_start(ap, fmt);
            vsnprintf(buf, len, fmt, ap);
            va_end(ap);
        }
        return st;
    }
};

static hc_status make_plan(const hc_config& cfg, const hc_head_desc* hd, int n_cu, int wg_per_cu, const float* share_weights,
                           Plan& P, const ErrBuf& E)
{
    const int nh = cfg.B * cfg.Hkv;
    const int max_reps = std::max(1, nh / 2);

    // ---- validate the head table ----
    for (int i = 0; i < nh; ++i) {
        const hc_head_desc& h = hd[i];
        if (h.role != HC_ROLE_FULL && h.role != HC_ROLE_SATELLITE && h.role != HC_ROLE_ANCHOR)
            return E.fail(HC_EINVAL, "head %d: bad role %d", i, h.role);
        if (h.cap != 0 && (h.cap < h.ctx || h.cap > cfg.max_ctx))
            return E.fail(HC_EINVAL, "head %d: cap %d outside ctx..max_ctx", i, h.cap);
        if (h.ctx < 1 || h.ctx > cfg.max_ctx) return E.fail(HC_ESHAPE, "head %d: ctx %d outside 1..%d", i, h.ctx, cfg.max_ctx);
        if (h.ctx != hd[i - i % cfg.Hkv].ctx) return E.fail(HC_EINVAL, "head %d: ctx differs within its sequence", i);
        if (h.len < 1 || h.len > h.ctx) return E.fail(HC_ESHAPE, "head %d: len %d outside 1..ctx", i, h.len);
        if (h.k_off < 0 || h.v_off < 0 || (h.k_off & 7) || (h.v_off & 7))
            return E.fail(HC_EINVAL, "head %d: k_off/v_off must be non-negative multiples of 8 elements", i);
        if (h.role == HC_ROLE_FULL) {
            if (h.len != h.ctx) return E.fail(HC_EINVAL, "head %d: a full head must have len == ctx", i);
            if (h.k_mon < 0) return E.fail(HC_EINVAL, "head %d: negative k_mon", i);
        } else {
            if (h.sink < 0 || h.recent < 0 || (int64_t)h.sink + h.recent > h.len)
                return E.fail(HC_EINVAL, "head %d: sink + recent exceeds its budget", i);
        }
        if (h.role == HC_ROLE_SATELLITE) {
            if (h.rep < 0 || h.rep >= cfg.Hkv || hd[i - i % cfg.Hkv + h.rep].role != HC_ROLE_FULL)
                return E.fail(HC_EINVAL, "head %d: rep %d is not a full head of the same sequence", i, h.rep);
            if (h.tier_off < 0 || (h.tier_off & 7)) return E.fail(HC_EINVAL, "head %d: bad tier_off", i);
        }
    }
    // K and V blocks of all heads must not overlap each other
    {
        std::vector<std::pair<int64_t, int64_t>> iv;
        for (int i = 0; i < nh; ++i) {
            const int64_t rows = hd[i].role == HC_ROLE_FULL && hd[i].cap > hd[i].len ? hd[i].cap : hd[i].len;
            iv.push_back({hd[i].k_off, hd[i].k_off + rows * HC_D});
            iv.push_back({hd[i].v_off, hd[i].v_off + rows * HC_D});
        }
        std::sort(iv.begin(), iv.end());
        for (size_t i = 1; i < iv.size(); ++i)
            if (iv[i].first < iv[i - 1].second) return E.fail(HC_EINVAL, "K/V blocks of two heads overlap in the arena");
    }

    // ---- pivots, their set sizes, the lists to emit, the satellites to refill ----
    P.rep_slot_of.assign(nh, -1);
    for (int b = 0; b < cfg.B; ++b) {
        for (int p = 0; p < cfg.Hkv; ++p) {
            const int pi = b * cfg.Hkv + p;
            std::vector<int> mine;
            for (int s = 0; s < cfg.Hkv; ++s) {
                const hc_head_desc& h = hd[b * cfg.Hkv + s];
                if (h.role == HC_ROLE_SATELLITE && h.rep == p) mine.push_back(b * cfg.Hkv + s);
            }
            if (mine.empty()) continue;
            RepDev r;
            memset(&r, 0, sizeof r);
            r.bh = pi;
            const hc_head_desc& s0 = hd[mine[0]];
            r.lo = s0.sink;
            r.hi = s0.ctx - s0.recent;
            int maxr = 0;
            for (int si : mine) {
                const hc_head_desc& h = hd[si];
                if (h.sink != s0.sink || h.recent != s0.recent)
                    return E.fail(HC_EINVAL, "pivot %d: its satellites must share sink and recent", pi);
                maxr = std::max(maxr, h.len - h.sink - h.recent);
            }
            const int kmon = hd[pi].k_mon > 0 ? hd[pi].k_mon : maxr;
            if (kmon < 1 || kmon > r.hi - r.lo || kmon > cfg.max_k)
                return E.fail(HC_EINVAL, "pivot %d: k_mon %d outside 1..min(candidates %d, max_k %d)", pi, kmon,
                              r.hi - r.lo, cfg.max_k);
            r.k[0] = kmon;
            r.nk = 1;
            const int slot = (int)P.reps.size();
            if (slot >= max_reps) return E.fail(HC_ESHAPE, "more pivots than the context was sized for");
            r.out_begin = (int32_t)P.outs.size();
            P.outs.push_back(OutDev{slot, 0, pi, 1});
            for (int si : mine) {
                const hc_head_desc& h = hd[si];
                const int rr = h.len - h.sink - h.recent;
                if (rr == 0) continue;
                if (rr > cfg.max_k) return E.fail(HC_EINVAL, "head %d: r %d exceeds max_k %d", si, rr, cfg.max_k);
                if (rr > r.hi - r.lo) return E.fail(HC_EINVAL, "head %d: more retrieved slots than candidate positions", si);
                int ks = -1;
                for (int t = 0; t < r.nk; ++t)
                    if (r.k[t] == rr) ks = t;
                if (ks < 0) {
                    if (r.nk == HC_MAX_K_PER_REP)
                        return E.fail(HC_ESHAPE, "pivot %d: more than %d distinct set sizes", pi, HC_MAX_K_PER_REP);
                    ks = r.nk++;
                    r.k[ks] = rr;
                }
                P.outs.push_back(OutDev{slot, ks, si, 0});
                P.sats.push_back(SatDev{si, pi, rr, h.sink + h.recent});
                P.max_r = std::max(P.max_r, rr);
            }
            r.out_count = (int32_t)P.outs.size() - r.out_begin;
            r.nchunk = (r.hi - r.lo + HC_SEL_CHUNK - 1) / HC_SEL_CHUNK;
            P.max_nchunk = std::max(P.max_nchunk, r.nchunk);
            P.rep_slot_of[pi] = slot;
            P.reps.push_back(r);
        }
    }

    // ---- split-K plan.  The rows of all heads, in granules of HC_UNIT_ROWS, are cut into equal
    // contiguous shares, one per workgroup; a share that crosses a head boundary becomes several
    // segments, each producing its own partial result.
    P.heads.resize(nh);
    const int64_t max_blocks = (int64_t)wg_per_cu * n_cu;
    const int64_t min_units = 4;
    int64_t total_units = 0;
    for (int i = 0; i < nh; ++i) {
        total_units += (hd[i].len + HC_UNIT_ROWS - 1) / HC_UNIT_ROWS;
        P.total_rows += hd[i].len;
        HeadDev& H = P.heads[i];
        H.k_off = hd[i].k_off;
        H.v_off = hd[i].v_off;
        H.tier_off = hd[i].tier_off;
        H.len = hd[i].len;
        H.ctx = hd[i].ctx;
        H.rep_slot = P.rep_slot_of[i];
        H.part_begin = 0;
        H.part_count = 0;
        H.role = hd[i].role;
        H.sink = hd[i].sink;
        H.recent = hd[i].recent;
        H.ctx0 = hd[i].ctx;
        H.tail_seg = H.tail_blk = -1;
        H.pad = 0;
    }
    const int nb = (int)std::max<int64_t>(1, std::min<int64_t>(max_blocks, total_units / min_units));
    P.n_blocks = nb;
    P.blk_seg.assign(nb + 1, 0);
    // Long passes whose workgroups come in whole groups of one per die and dispatch slot get shares
    // weighted by the class the share runs on (share l runs on die (l % 16) / 2, slot l % 2).
    const bool weighted = share_weights != nullptr && nb % 16 == 0 && total_units >= 16 * (int64_t)nb;   // >= 512 rows per workgroup

    std::vector<int64_t> head_first(nh + 1, 0);        // first granule of every head
    for (int i = 0; i < nh; ++i) head_first[i + 1] = head_first[i] + (hd[i].len + HC_UNIT_ROWS - 1) / HC_UNIT_ROWS;
    auto head_of_unit = [&](int64_t u) {
        return (int)(std::upper_bound(head_first.begin(), head_first.end(), u) - head_first.begin()) - 1;
    };

    // Shares are cut on a cost axis: one per granule, plus SEG_COST granules at every head boundary, because a
    // workgroup whose share crosses a boundary closes one state (merge of its waves, partial result
    // written) and opens another (new query rows, load pipeline refilled), which costs it the time of
    // about 100 rows.  cost_start[h] is where head h's boundary cost begins; its granules follow it.
    // (Measured at the 224K shape: the workgroups that cross a boundary were the last to finish by 2 us.)
    const int64_t SEG_COST = total_units >= 16 * (int64_t)nb ? 3 : 0;
    std::vector<int64_t> cost_start(nh + 1, 0);
    for (int i = 1; i <= nh; ++i) cost_start[i] = head_first[i] + SEG_COST * (i - 1);
    const int64_t total_cost = cost_start[nh];            // = total_units + SEG_COST * (nh - 1)
    auto unit_of_cost = [&](int64_t cst) {                 // first granule at or after this point of the cost axis
        if (cst >= total_cost) return total_units;
        const int h = (int)(std::upper_bound(cost_start.begin(), cost_start.begin() + nh, cst) - cost_start.begin()) - 1;
        const int64_t into = cst - cost_start[h] - (h > 0 ? SEG_COST : 0);
        return head_first[h] + std::max<int64_t>(0, into);
    };

    // share boundaries [lo, hi) in granules
    std::vector<int64_t> lo(nb), hi(nb);
    {
        double total_w = 0;
        for (int l = 0; l < nb; ++l) total_w += weighted ? share_weights[l % 16] : 1.0;
        double acc_w = 0;
        int64_t prev = 0;
        for (int l = 0; l < nb; ++l) {
            acc_w += weighted ? share_weights[l % 16] : 1.0;
            int64_t end = l + 1 == nb ? total_units : unit_of_cost((int64_t)((double)total_cost * acc_w / total_w + 0.5));
            end = std::min(std::max(end, prev), total_units);
            lo[l] = prev;
            hi[l] = end;
            prev = end;
        }
    }

    // segments of the shares, one partial-result slot each
    for (int blk = 0; blk < nb; ++blk) {
        int64_t u0 = lo[blk];
        const int64_t u1 = hi[blk];
        P.blk_seg[blk] = (int32_t)P.segs.size();
        while (u0 < u1) {
            const int head = head_of_unit(u0);
            const int64_t take_end = std::min(u1, head_first[head + 1]);
            SegDev sg;
            sg.k_off = hd[head].k_off;
            sg.v_off = hd[head].v_off;
            sg.rep_slot = P.rep_slot_of[head];
            sg.pad = 0;
            sg.bh = head;
            sg.row_begin = (int32_t)((u0 - head_first[head]) * HC_UNIT_ROWS);
            sg.row_end = (int32_t)std::min<int64_t>((take_end - head_first[head]) * HC_UNIT_ROWS, hd[head].len);
            sg.slot = (int32_t)P.segs.size();
            if (P.heads[head].part_count == 0) P.heads[head].part_begin = sg.slot;
            P.heads[head].part_count++;
            P.segs.push_back(sg);
            u0 = take_end;
        }
    }
    P.blk_seg[nb] = (int32_t)P.segs.size();
    for (int blk = 0; blk < nb; ++blk)
        if (P.blk_seg[blk] == P.blk_seg[blk + 1]) return E.fail(HC_ESTATE, "internal: workgroup %d has no rows", blk);

    // Placement.  On MI355X a workgroup's index modulo 8 is the die (XCD) it runs on, and with two
    // workgroups per compute unit the second half of the indices are the second ones dispatched; dies
    // and dispatch slots stream at measurably different speeds.  Share l = 16 j + 2 x + slot runs as
    // workgroup slot * nb/2 + 8 j + x, so that neighbouring stretches of rows (in particular the two
    // ends of a head) are spread over all dies and both slots instead of falling on the same kind.
    P.blks.resize(nb);
    for (int l = 0; l < nb; ++l) {
        int p = l;
        if (nb % 16 == 0) p = (l % 2) * (nb / 2) + (l / 16) * 8 + (l % 16) / 2;
        BlkDev& B = P.blks[p];
        B.first = P.segs[P.blk_seg[l]];
        B.extra_begin = P.blk_seg[l] + 1;
        B.extra_end = P.blk_seg[l + 1];
        B.pad0 = B.pad1 = 0;
        // a full head's last segment grows with appended tokens: remember where its copies live
        for (int sg = P.blk_seg[l]; sg < P.blk_seg[l + 1]; ++sg) {
            HeadDev& H = P.heads[P.segs[sg].bh];
            if (hd[P.segs[sg].bh].role == HC_ROLE_FULL && P.segs[sg].row_end == hd[P.segs[sg].bh].len) {
                H.tail_seg = sg;
                H.tail_blk = sg == P.blk_seg[l] ? p : -1;
            }
        }
    }
    return HC_OK;
}

extern "C" hc_status hc_plan_describe(const hc_config* cfg, const hc_head_desc* heads_host, int32_t compute_units,
                                      int32_t workgroups_per_cu, hc_plan_info* info, char* err, int32_t err_len)
{
    if (err && err_len > 0) err[0] = 0;
    if (!cfg || !heads_host || !info) return HC_EINVAL;
    const hc_status cs = check_config(cfg);
    if (cs != HC_OK) return cs;
    if (compute_units < 1 || compute_units > 4096 || workgroups_per_cu < 1 || workgroups_per_cu > 16) return HC_EINVAL;
    Plan P;
    const hc_status st = make_plan(*cfg, heads_host, compute_units, workgroups_per_cu, DEFAULT_SHARE_WEIGHTS, P,
                                   ErrBuf{err, err_len > 0 ? (size_t)err_len : 0});
    if (st != HC_OK) return st;
    memset(info, 0, sizeof *info);
    info->n_workgroups = P.n_blocks;
    info->n_partials = (int32_t)P.segs.size();
    info->n_reps = (int32_t)P.reps.size();
    info->n_lists = (int32_t)P.outs.size();
    info->n_satellites = (int32_t)P.sats.size();
    info->total_rows = P.total_rows;
    info->min_rows_per_workgroup = INT32_MAX;
    std::vector<int64_t> covered(cfg->B * cfg->Hkv, 0);
    for (int b = 0; b < P.n_blocks; ++b) {
        int rows = 0;
        for (int s = P.blk_seg[b]; s < P.blk_seg[b + 1]; ++s) {
            rows += P.segs[s].row_end - P.segs[s].row_begin;
            covered[P.segs[s].bh] += P.segs[s].row_end - P.segs[s].row_begin;
        }
        info->max_rows_per_workgroup = std::max(info->max_rows_per_workgroup, rows);
        info->min_rows_per_workgroup = std::min(info->min_rows_per_workgroup, rows);
    }
    info->rows_covered = 0;
    for (int i = 0; i < cfg->B * cfg->Hkv; ++i)
        if (covered[i] == heads_host[i].len) info->rows_covered += covered[i];
    return HC_OK;
}

extern "C" hc_status hc_layer_create(hc_ctx* ctx, const hc_head_desc* hd, hc_layer** out)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    if (!hd || !out) return hc_fail(ctx, HC_EINVAL, "hc_layer_create: null argument");
    *out = nullptr;
    Plan P;
    hc_status st = make_plan(ctx->cfg, hd, ctx->n_cu, ctx->wg_per_cu, ctx->share_weights, P, ErrBuf{ctx->err, sizeof ctx->err});
    if (st != HC_OK) return st;

    hc_layer* L = new (std::nothrow) hc_layer();
    if (!L) return hc_fail(ctx, HC_ENOMEM, "host allocation failed");
    L->magic = HC_LAYER_MAGIC;
    L->ctx = ctx;
    L->n_heads = ctx->cfg.B * ctx->cfg.Hkv;
    L->rep_slot_of = P.rep_slot_of;
    L->max_r = P.max_r;
    L->max_nchunk = P.max_nchunk;
    L->max_nk = 1;
    for (const RepDev& r : P.reps) {
        L->max_nk = std::max(L->max_nk, r.nk);
        for (int t = 0; t < r.nk; ++t) L->max_k_any = std::max(L->max_k_any, r.k[t]);
    }
    L->n_reps = (int)P.reps.size();
    L->n_outs = (int)P.outs.size();
    L->n_sats = (int)P.sats.size();
    L->n_blocks = P.n_blocks;
    L->n_segs = L->n_partials = (int)P.segs.size();
    L->hd_host.assign(hd, hd + L->n_heads);
    for (int i = 0; i < L->n_heads; ++i) L->ctx0_host.push_back(hd[i].ctx);
    for (const RepDev& r : P.reps) {
        L->rep_lo_host.push_back(r.lo);
        L->rep_recent_host.push_back(hd[r.bh].ctx - r.hi);
    }
    // a plan has at most one segment per workgroup plus one per head boundary, and a short layer gets more
    // workgroups as it grows: room for any later plan
    L->blk_capacity = ctx->wg_per_cu * ctx->n_cu;
    L->seg_capacity = L->blk_capacity + L->n_heads;

    st = ensure_partials(ctx, (size_t)L->seg_capacity);
    if (st == HC_OK) st = upload(ctx, P.heads, &L->heads);
    if (st == HC_OK) st = upload(ctx, P.segs, &L->segs, (size_t)L->seg_capacity);
    if (st == HC_OK) st = upload(ctx, P.blks, &L->blks, (size_t)L->blk_capacity);
    if (st == HC_OK) st = upload(ctx, P.reps, &L->reps);
    if (st == HC_OK) st = upload(ctx, P.outs, &L->outs);
    if (st == HC_OK) st = upload(ctx, P.sats, &L->sats);
    if (st == HC_OK) {
        // prefill-time selection (hc_prefill_init): every compressed head with refillable slots selects r
        // positions of its own candidates; every pivot selects its baseline set
        std::vector<RepDev> sel;
        std::vector<OutDev> outs;
        for (int i = 0; i < L->n_heads; ++i) {
            const hc_head_desc& h = hd[i];
            RepDev r;
            memset(&r, 0, sizeof r);
            r.bh = i;
            if (h.role == HC_ROLE_FULL) {
                if (P.rep_slot_of[i] < 0) continue;
                const RepDev& pv = P.reps[P.rep_slot_of[i]];
                r.lo = pv.lo;
                r.hi = pv.hi;
                r.k[0] = pv.k[0];
            } else {
                r.lo = h.sink;
                r.hi = h.ctx - h.recent;
                r.k[0] = h.len - h.sink - h.recent;
                if (r.k[0] == 0) continue;
                if (r.k[0] > ctx->cfg.max_k || r.k[0] > r.hi - r.lo) {
                    // fine for decoding (an anchor's slots are never selected again), but hc_prefill_init cannot fill them
                    L->prefill_unfit_head = i;
                    continue;
                }
            }
            r.nk = 1;
            r.nchunk = (r.hi - r.lo + HC_SEL_CHUNK - 1) / HC_SEL_CHUNK;
            r.out_begin = (int32_t)outs.size();
            r.out_count = 1;
            outs.push_back(OutDev{(int32_t)sel.size(), 0, i, 0});
            sel.push_back(r);
            L->sel_head_host.push_back(i);
            L->sel_max_nchunk = std::max(L->sel_max_nchunk, r.nchunk);
            L->sel_max_len = std::max(L->sel_max_len, (int)h.ctx);
        }
        L->n_sel = (int)sel.size();
        if (st == HC_OK) st = upload(ctx, sel, &L->sel_reps);
        if (st == HC_OK) st = upload(ctx, outs, &L->sel_outs);
        if (st == HC_OK) st = upload(ctx, std::vector<PreSrc>(), &L->pre_src, (size_t)L->n_heads);
        if (st == HC_OK) st = upload(ctx, P.rep_slot_of, &L->rep_slot_dev);
    }
    if (st == HC_OK && L->n_reps > 0) {
        // per-pivot counters of the monitor (tests, triggers, ...), read back by hc_layer_monitor_counts
        if (hipMalloc((void**)&L->mon_counts, (size_t)L->n_reps * 4 * sizeof(uint32_t)) != hipSuccess ||
            hipMemset(L->mon_counts, 0, (size_t)L->n_reps * 4 * sizeof(uint32_t)) != hipSuccess)
            st = hc_fail(ctx, HC_ENOMEM, "monitor counters");
    }
    int widest = 0;                                  // the longest candidate range of any pivot of the layer
    for (const RepDev& r : P.reps) widest = std::max(widest, r.hi - r.lo);
    if (st == HC_OK && ctx->filter_margin > 0.f && L->n_reps > 0 && L->blk_capacity < 2048 && widest >= ctx->filter_min_candidates) {
        // the pivot-logit filter's buffers (a split pass of 2048 or more workgroups keeps the plain form)
        const size_t nr = (size_t)L->n_reps, mc = (size_t)ctx->cfg.max_ctx;
        hipError_t e = hipMalloc((void**)&L->filt, nr * sizeof(RepFilter));
        if (e == hipSuccess) e = hipMemset(L->filt, 0, nr * sizeof(RepFilter));
        if (e == hipSuccess) e = hipMalloc((void**)&L->surv_pos, nr * mc * sizeof(int32_t));
        if (e == hipSuccess) e = hipMalloc((void**)&L->dense_pos, nr * mc * sizeof(int32_t));
        if (e == hipSuccess) e = hipMalloc((void**)&L->seg_cnt, (size_t)L->seg_capacity * sizeof(int32_t));
        if (e == hipSuccess) e = hipMemset(L->seg_cnt, 0, (size_t)L->seg_capacity * sizeof(int32_t));
        if (e == hipSuccess) e = hipMalloc((void**)&L->vreps, nr * sizeof(RepDev));
        if (e == hipSuccess) e = hipMemcpy(L->vreps, P.reps.data(), nr * sizeof(RepDev), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMalloc((void**)&L->need, nr * sizeof(int32_t));
        if (e == hipSuccess) e = hipMemset(L->need, 0, nr * sizeof(int32_t));
        if (e == hipSuccess) e = hipMalloc((void**)&L->q_keep, nr * ctx->G * HC_D * sizeof(uint16_t));
        if (e == hipSuccess) e = hipMemset(L->q_keep, 0, nr * ctx->G * HC_D * sizeof(uint16_t));
        if (e != hipSuccess) st = hc_hip_fail(ctx, e, "buffers of the pivot-logit filter");
    }
    if (st == HC_OK) {
        // staging for rebalanced plans: heads, segments, workgroup descriptors, pivots, each 16-byte aligned
        auto up16 = [](size_t x) { return (x + 15) & ~(size_t)15; };
        L->plan_stage_bytes = up16((size_t)L->n_heads * sizeof(HeadDev)) + up16((size_t)L->seg_capacity * sizeof(SegDev)) +
                              up16((size_t)L->blk_capacity * sizeof(BlkDev)) + up16((size_t)std::max(1, L->n_reps) * sizeof(RepDev));
        for (int i = 0; i < 2 && st == HC_OK; ++i) {
            if (hipHostMalloc((void**)&L->plan_stage[i], L->plan_stage_bytes, hipHostMallocDefault) != hipSuccess)
                st = hc_fail(ctx, HC_ENOMEM, "pinned staging for the split-K plan");
            else if (hipEventCreateWithFlags(&L->plan_copied[i], hipEventDisableTiming) != hipSuccess)
                st = hc_fail(ctx, HC_EHIP, "hipEventCreate failed");
        }
    }
    if (st == HC_OK && hipEventCreateWithFlags(&L->ev_attn, hipEventDisableTiming) != hipSuccess) st = hc_fail(ctx, HC_EHIP, "hipEventCreate failed");
    if (st == HC_OK && hipEventCreateWithFlags(&L->ev_side, hipEventDisableTiming) != hipSuccess) st = hc_fail(ctx, HC_EHIP, "hipEventCreate failed");
    if (st != HC_OK) {
        layer_free(L);
        return st;
    }
    *out = L;
    return HC_OK;
}

extern "C" hc_status hc_layer_destroy(hc_layer* layer)
{
    if (!layer_ok(layer)) return HC_ESTATE;
    layer_free(layer);
    return HC_OK;
}

extern "C" int32_t hc_layer_num_reps(const hc_layer* layer) { return layer_ok(layer) ? layer->n_reps : -1; }
extern "C" int32_t hc_layer_num_workgroups(const hc_layer* layer) { return layer_ok(layer) ? layer->n_blocks : -1; }
extern "C" int32_t hc_layer_num_partials(const hc_layer* layer) { return layer_ok(layer) ? layer->n_partials : -1; }

extern "C" int32_t hc_layer_rep_slot(const hc_layer* layer, int32_t b, int32_t h)
{
    if (!layer_ok(layer)) return -1;
    const hc_config& c = layer->ctx->cfg;
    if (b < 0 || b >= c.B || h < 0 || h >= c.Hkv) return -1;
    return layer->rep_slot_of[b * c.Hkv + h];
}

// ---- hot path: validate, then enqueue ------------------------------------------------------
static hc_status attn_check(hc_ctx* ctx, const hc_layer* layer, const void* kv_arena, const void* q, const float* out, const float* lse,
                            const float* rep_logits);

extern "C" hc_status hc_decode_attn(hc_ctx* ctx, const hc_layer* layer, const void* kv_arena, const void* q,
                                    float* out, float* lse, float* rep_logits, void* stream)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    const hc_status chk = attn_check(ctx, layer, kv_arena, q, out, lse, rep_logits);
    if (chk != HC_OK) return chk;
    if (rep_logits) const_cast<hc_layer*>(layer)->last_arena = kv_arena;
    return hc_launch_attn(ctx, layer, kv_arena, q, out, lse, rep_logits, (hipStream_t)stream);
}

extern "C" hc_status hc_decode_attn_static(hc_ctx* ctx, const hc_layer* layer, const void* kv_arena, const void* q,
                                           float* out, float* lse, float* rep_logits, void* stream)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    const hc_status chk = attn_check(ctx, layer, kv_arena, q, out, lse, rep_logits);
    if (chk != HC_OK) return chk;
    if (rep_logits) const_cast<hc_layer*>(layer)->last_arena = kv_arena;
    return hc_launch_attn_static(ctx, layer, kv_arena, q, out, lse, rep_logits, (hipStream_t)stream);
}

static hc_status monitor_check(hc_ctx* ctx, const hc_layer* layer, const float* rep_logits, const float* lse,
                               const float* scores, int32_t scores_given, const int32_t* topk_idx,
                               const int32_t* base_idx, const int32_t* ring, const int32_t* inter, const int32_t* flag)
{
    if (!layer_ok(layer) || layer->ctx != ctx) return hc_fail(ctx, HC_ESTATE, "hc_rep_topk_drift: layer does not belong to this context");
    if (!scores || !topk_idx || !base_idx || !ring || !inter || !flag)
        return hc_fail(ctx, HC_EINVAL, "hc_rep_topk_drift: null pointer");
    if (!scores_given && (!rep_logits || (ctx->cfg.agg == HC_AGG_PROB && !lse)))
        return hc_fail(ctx, HC_EINVAL, "hc_rep_topk_drift: rep_logits and lse are needed unless scores are given");
    if (((uintptr_t)scores | (uintptr_t)rep_logits) & 15)
        return hc_fail(ctx, HC_EINVAL, "hc_rep_topk_drift: scores and rep_logits must be 16-byte aligned");
    return HC_OK;
}

extern "C" hc_status hc_rep_topk_drift(hc_ctx* ctx, const hc_layer* layer, const float* rep_logits, const float* lse,
                                       float* scores, int32_t scores_given, int32_t* topk_idx, int32_t* base_idx,
                                       int32_t* ring, int32_t* inter, int32_t* flag, void* stream)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    const hc_status st = monitor_check(ctx, layer, rep_logits, lse, scores, scores_given, topk_idx, base_idx, ring, inter, flag);
    if (st != HC_OK) return st;
    if (layer->n_reps == 0) return HC_OK;
    const hc_monitor_call call{layer, rep_logits, lse, scores, topk_idx, base_idx, ring, inter, flag};
    return hc_launch_monitor(ctx, 1, &call, scores_given != 0, (hipStream_t)stream);
}

static hc_status gather_check(hc_ctx* ctx, const hc_layer* layer, const void* host_tier, const int32_t* topk_idx,
                              const int32_t* flag, const void* kv_arena)
{
    if (!layer_ok(layer) || layer->ctx != ctx) return hc_fail(ctx, HC_ESTATE, "hc_gather_retrieve: layer does not belong to this context");
    if (!topk_idx || !flag || !kv_arena || (!host_tier && layer->n_sats > 0))
        return hc_fail(ctx, HC_EINVAL, "hc_gather_retrieve: null pointer");
    if (((uintptr_t)kv_arena | (uintptr_t)host_tier) & 15)
        return hc_fail(ctx, HC_EINVAL, "hc_gather_retrieve: kv_arena and host_tier must be 16-byte aligned");
    return HC_OK;
}

extern "C" hc_status hc_gather_retrieve(hc_ctx* ctx, const hc_layer* layer, const void* host_tier,
                                        const int32_t* topk_idx, const int32_t* flag, void* kv_arena,
                                        int32_t* slot_pos, void* stream, void* wait_event, void* done_event)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    const hc_status chk = gather_check(ctx, layer, host_tier, topk_idx, flag, kv_arena);
    if (chk != HC_OK) return chk;
    hipStream_t st = (hipStream_t)stream;
    if (wait_event) HC_HIP(ctx, hipStreamWaitEvent(st, (hipEvent_t)wait_event, 0));
    if (layer->n_sats > 0) {
        const hc_gather_call call{layer, host_tier, topk_idx, flag, kv_arena, slot_pos};
        const hc_status s = hc_launch_gather(ctx, 1, &call, st);
        if (s != HC_OK) return s;
    }
    if (done_event) HC_HIP(ctx, hipEventRecord((hipEvent_t)done_event, st));
    return HC_OK;
}

extern "C" hc_status hc_layer_monitor_counts(const hc_layer* layer, int32_t b, int32_t h, uint32_t* counts4)
{
    if (!layer_ok(layer)) return HC_ESTATE;
    const hc_config& c = layer->ctx->cfg;
    if (!counts4 || b < 0 || b >= c.B || h < 0 || h >= c.Hkv || layer->rep_slot_of[b * c.Hkv + h] < 0 || !layer->mon_counts)
        return hc_fail(layer->ctx, HC_EINVAL, "hc_layer_monitor_counts: (b, h) is not a pivot of this layer");
    HC_HIP(layer->ctx, hipMemcpy(counts4, layer->mon_counts + (size_t)layer->rep_slot_of[b * c.Hkv + h] * 4, 4 * sizeof(uint32_t),
                                 hipMemcpyDeviceToHost));
    return HC_OK;
}

extern "C" hc_status hc_layer_filter_view(const hc_layer* layer, const int32_t** kept_pos, const int32_t** fell_back)
{
    if (!layer_ok(layer)) return HC_ESTATE;
    if (kept_pos) *kept_pos = layer->dense_pos;
    if (fell_back) *fell_back = layer->need;
    return HC_OK;
}

extern "C" int32_t hc_layer_context(const hc_layer* layer, int32_t b)
{
    if (!layer_ok(layer) || b < 0 || b >= layer->ctx->cfg.B) return -1;
    return layer->hd_host[(size_t)b * layer->ctx->cfg.Hkv].ctx;
}

// Rebuilds the split-K plan from the head table as it is now and copies it over the old one on `st`.
// The workgroup count and the pivots do not change with the lengths; only shares, segments and slots do.
// Enqueue-only: the new tables are written into one of the layer's two pinned staging buffers and copied
// from there in stream order (behind the append kernel whose lengths they include, ahead of the attention
// that uses them).  The host waits only if the buffer's previous copy, two rebalancings ago, has not run yet.
static hc_status replan(hc_ctx* ctx, hc_layer* L, hipStream_t st)
{
    Plan P;
    hc_status s = make_plan(ctx->cfg, L->hd_host.data(), ctx->n_cu, ctx->wg_per_cu, ctx->share_weights, P,
                            ErrBuf{ctx->err, sizeof ctx->err});
    if (s != HC_OK) return s;
    if (P.n_blocks > L->blk_capacity || (int)P.segs.size() > L->seg_capacity || (int)P.reps.size() != L->n_reps)
        return hc_fail(ctx, HC_ESTATE, "internal: a rebalanced plan does not fit the layer");
    for (int i = 0; i < L->n_heads; ++i) P.heads[i].ctx0 = L->ctx0_host[i];        // the ring of recent slots keeps its origin
    auto up16 = [](size_t x) { return (x + 15) & ~(size_t)15; };
    const size_t b_heads = P.heads.size() * sizeof(HeadDev), b_segs = P.segs.size() * sizeof(SegDev),
                 b_blks = P.blks.size() * sizeof(BlkDev), b_reps = P.reps.size() * sizeof(RepDev);
    const size_t o_segs = up16(b_heads), o_blks = o_segs + up16(b_segs), o_reps = o_blks + up16(b_blks);
    if (o_reps + b_reps > L->plan_stage_bytes) return hc_fail(ctx, HC_ESTATE, "internal: plan staging too small");
    const int which = L->plan_next;
    L->plan_next ^= 1;
    HC_HIP(ctx, hipEventSynchronize(L->plan_copied[which]));       // (an event never recorded counts as complete)
    char* stage = L->plan_stage[which];
    memcpy(stage, P.heads.data(), b_heads);
    memcpy(stage + o_segs, P.segs.data(), b_segs);
    memcpy(stage + o_blks, P.blks.data(), b_blks);
    if (b_reps) memcpy(stage + o_reps, P.reps.data(), b_reps);
    HC_HIP(ctx, hipMemcpyAsync(L->heads, stage, b_heads, hipMemcpyHostToDevice, st));
    HC_HIP(ctx, hipMemcpyAsync(L->segs, stage + o_segs, b_segs, hipMemcpyHostToDevice, st));
    HC_HIP(ctx, hipMemcpyAsync(L->blks, stage + o_blks, b_blks, hipMemcpyHostToDevice, st));
    if (b_reps) HC_HIP(ctx, hipMemcpyAsync(L->reps, stage + o_reps, b_reps, hipMemcpyHostToDevice, st));
    HC_HIP(ctx, hipEventRecord(L->plan_copied[which], st));
    L->n_blocks = P.n_blocks;
    L->n_segs = L->n_partials = (int)P.segs.size();
    L->max_nchunk = P.max_nchunk;
    L->appended_since_plan = 0;
    return HC_OK;
}

static hc_status append_check(hc_ctx* ctx, const hc_layer* layer, const void* k_new, const void* v_new, const void* kv_arena,
                              const void* host_tier)
{
    if (!layer_ok(layer) || layer->ctx != ctx) return hc_fail(ctx, HC_ESTATE, "hc_append_kv: layer does not belong to this context");
    if (!k_new || !v_new || !kv_arena) return hc_fail(ctx, HC_EINVAL, "hc_append_kv: null pointer");
    if (((uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)kv_arena | (uintptr_t)host_tier) & 3)
        return hc_fail(ctx, HC_EINVAL, "hc_append_kv: pointers must be 4-byte aligned");
    for (int i = 0; i < layer->n_heads; ++i) {
        const hc_head_desc& h = layer->hd_host[i];
        const bool grows = h.role == HC_ROLE_FULL || h.role == HC_ROLE_SATELLITE;
        if (h.ctx + 1 > ctx->cfg.max_ctx || (grows && h.ctx + 1 > (h.cap ? h.cap : h.ctx)))
            return hc_fail(ctx, HC_ESHAPE, "hc_append_kv: head %d has no room for position %d (cap %d, max_ctx %d)", i, h.ctx,
                           h.cap, ctx->cfg.max_ctx);
        if (h.role == HC_ROLE_SATELLITE && !host_tier) return hc_fail(ctx, HC_EINVAL, "hc_append_kv: host_tier is needed for satellites");
    }
    return HC_OK;
}

// The host's copy of the lengths follows what the kernel does to the device tables; every 64 tokens the
// split-K plan is rebalanced.
static hc_status append_done(hc_ctx* ctx, hc_layer* L, hipStream_t st)
{
    for (int i = 0; i < L->n_heads; ++i) {
        hc_head_desc& h = L->hd_host[i];
        h.ctx += 1;
        if (h.role == HC_ROLE_FULL) h.len += 1;
    }
    int max_nchunk = 1;
    for (int i = 0; i < L->n_heads; ++i)
        if (L->rep_slot_of[i] >= 0) {
            const int slot = L->rep_slot_of[i];
            const int lo = L->rep_lo_host[slot], hi = L->hd_host[i].ctx - L->rep_recent_host[slot];
            max_nchunk = std::max(max_nchunk, (hi - lo + HC_SEL_CHUNK - 1) / HC_SEL_CHUNK);
        }
    L->max_nchunk = max_nchunk;
    ++L->total_appended;
    if (++L->appended_since_plan >= 64) return replan(ctx, L, st);
    return HC_OK;
}

extern "C" hc_status hc_append_kv(hc_ctx* ctx, hc_layer* layer, const void* k_new, const void* v_new, void* kv_arena,
                                  void* host_tier, void* stream)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    hc_status s = append_check(ctx, layer, k_new, v_new, kv_arena, host_tier);
    if (s != HC_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    const hc_append_call call{layer, k_new, v_new, kv_arena, host_tier};
    s = hc_launch_append(ctx, 1, &call, st);
    if (s != HC_OK) return s;
    return append_done(ctx, layer, st);
}

// Share weights measured on the device at hand.  Which dies stream slower differs from one MI355X to the
// next (and the built-in weights come from one of them), so the layer's own split pass is run a few times
// with per-workgroup timestamps, the 16 (die, dispatch slot) classes' mean finish times are equalised
// (work_c proportional to rate_c * (T - entry_c)), and the layer is replanned; the weights stay in the
// context for the layers created afterwards.  Launches are timed back to back, as in a decode step: a
// launch into an idle GPU reaches the dies up to 2 us apart, which steady state does not see.
extern "C" hc_status hc_layer_tune(hc_ctx* ctx, hc_layer* layer, const void* kv_arena, const void* q, float* out, float* lse,
                                   float* rep_logits, int32_t rounds, void* stream)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    if (!layer_ok(layer) || layer->ctx != ctx) return hc_fail(ctx, HC_ESTATE, "hc_layer_tune: layer does not belong to this context");
    if (rounds < 1 || rounds > 16) return hc_fail(ctx, HC_EINVAL, "hc_layer_tune: rounds 1..16");
    hc_layer* L = layer;
    const int nb = L->n_blocks;
    int64_t total_units = 0;
    for (const hc_head_desc& h : L->hd_host) total_units += (h.len + HC_UNIT_ROWS - 1) / HC_UNIT_ROWS;
    if (nb % 16 != 0 || total_units < 16 * (int64_t)nb) return HC_OK;        // shares of this plan are not weighted
    hipStream_t st = (hipStream_t)stream;
    unsigned long long* dev = nullptr;
    HC_HIP(ctx, hipMalloc((void**)&dev, (size_t)nb * 2 * sizeof(unsigned long long)));
    std::vector<unsigned long long> host((size_t)nb * 2);
    hc_status result = HC_OK;
    constexpr int SAMPLES = 6;
    for (int round = 0; round < rounds && result == HC_OK; ++round) {
        double ent[16] = {}, fin[16] = {};
        bool give_up = false;
        for (int s = 0; s < SAMPLES && result == HC_OK; ++s) {
            for (int k = 0; k < 3 && result == HC_OK; ++k) {                  // the third of three back-to-back launches is read
                ctx->tune_stamps = k == 2 ? dev : nullptr;
                if (k == 2 && hipMemsetAsync(dev, 0, host.size() * sizeof(unsigned long long), st) != hipSuccess) result = HC_EHIP;
                if (result == HC_OK) result = hc_decode_attn(ctx, L, kv_arena, q, out, lse, rep_logits, st);
            }
            ctx->tune_stamps = nullptr;
            if (result != HC_OK) break;
            hipError_t e = hipStreamSynchronize(st);
            if (e == hipSuccess) e = hipMemcpy(host.data(), dev, host.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost);
            if (e != hipSuccess) {
                result = hc_hip_fail(ctx, e, "hc_layer_tune");
                break;
            }
            unsigned long long t0 = ~0ull;
            bool stamped = true;
            for (int b = 0; b < nb; ++b) {
                t0 = std::min(t0, host[2 * b]);
                stamped &= host[2 * b] != 0 && host[2 * b + 1] > host[2 * b];
            }
            if (!stamped) {                                                    // a workgroup left no time: keep what we have
                give_up = true;
                break;
            }
            for (int b = 0; b < nb; ++b) {
                const int cls = (b % 8) * 2 + (b >= nb / 2);
                ent[cls] += (double)(host[2 * b] - t0) / (nb / 16) / SAMPLES;
                fin[cls] += (double)(host[2 * b + 1] - t0) / (nb / 16) / SAMPLES;
            }
        }
        if (result != HC_OK || give_up) break;
        double rate[16], sum_w = 0, sum_rate = 0, sum_re = 0;
        bool ok = true;
        for (int c = 0; c < 16; ++c) {
            ok &= fin[c] > ent[c];
            rate[c] = ctx->share_weights[c] / std::max(1.0, fin[c] - ent[c]);
            sum_w += ctx->share_weights[c];
            sum_rate += rate[c];
            sum_re += rate[c] * ent[c];
        }
        if (!ok) break;                                                        // timestamps make no sense: keep what we have
        const double T = (sum_w + sum_re) / sum_rate;
        double neww[16], sum_new = 0;
        for (int c = 0; c < 16; ++c) {
            neww[c] = rate[c] * (T - ent[c]);
            sum_new += neww[c];
        }
        for (int c = 0; c < 16; ++c) {
            const double w = 0.5 * ctx->share_weights[c] + 0.5 * neww[c] * 16.0 / sum_new;      // damped
            ctx->share_weights[c] = (float)std::min(1.25, std::max(0.8, w));
        }
        result = replan(ctx, L, st);
    }
    ctx->tune_stamps = nullptr;
    (void)hipFree(dev);
    return result;
}

// ---- prefill-time initialisation (Sec. 4.3; Algorithm 1, stage 3 before the loop) ----
extern "C" size_t hc_prefill_work_bytes(const hc_ctx* ctx, const hc_layer* layer)
{
    if (!ctx_ok(ctx) || !layer_ok(layer) || layer->ctx != ctx) return 0;
    return hc_prefill_plan(ctx, layer).bytes;
}

extern "C" hc_status hc_prefill_work_layout(const hc_ctx* ctx, const hc_layer* layer, int32_t* n_selecting, int32_t* head_of,
                                            size_t* logits_off, size_t* scores_off, size_t* lse_off)
{
    if (!ctx_ok(ctx) || !layer_ok(layer) || layer->ctx != ctx) return HC_ESTATE;
    const hc_prefill_layout lay = hc_prefill_plan(ctx, layer);
    if (n_selecting) *n_selecting = layer->n_sel;
    if (head_of)
        for (int i = 0; i < layer->n_sel; ++i) head_of[i] = layer->sel_head_host[(size_t)i];
    if (logits_off) *logits_off = lay.logits_off;
    if (scores_off) *scores_off = lay.scores_off;
    if (lse_off) *lse_off = lay.lse_off;
    return HC_OK;
}

extern "C" hc_status hc_prefill_init(hc_ctx* ctx, hc_layer* layer, const void* kv_prefill, const int64_t* k_src_off,
                                     const int64_t* v_src_off, const void* q_last, int32_t pool, void* kv_arena, void* host_tier,
                                     int32_t* topk_idx, int32_t* base_idx, int32_t* slot_pos, int32_t* ring, void* work,
                                     size_t work_bytes, void* stream)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    if (!layer_ok(layer) || layer->ctx != ctx) return hc_fail(ctx, HC_ESTATE, "hc_prefill_init: layer does not belong to this context");
    hc_layer* L = layer;
    if (!kv_prefill || !k_src_off || !v_src_off || !q_last || !kv_arena || !topk_idx || !base_idx || !ring || !work)
        return hc_fail(ctx, HC_EINVAL, "hc_prefill_init: null pointer");
    if (pool < 1 || pool > HC_MAX_POOL || pool % 2 == 0) return hc_fail(ctx, HC_EINVAL, "hc_prefill_init: pool %d must be odd, 1..%d", (int)pool, HC_MAX_POOL);
    if (((uintptr_t)kv_prefill | (uintptr_t)kv_arena | (uintptr_t)host_tier | (uintptr_t)q_last) & 15)
        return hc_fail(ctx, HC_EINVAL, "hc_prefill_init: buffers must be 16-byte aligned");
    if ((uintptr_t)work & 255) return hc_fail(ctx, HC_EINVAL, "hc_prefill_init: work must be 256-byte aligned");
    const hc_prefill_layout lay = hc_prefill_plan(ctx, L);
    if (work_bytes < lay.bytes) return hc_fail(ctx, HC_EINVAL, "hc_prefill_init: work buffer of %zu bytes, %zu needed", work_bytes, lay.bytes);
    if (L->total_appended != 0) return hc_fail(ctx, HC_ESTATE, "hc_prefill_init: tokens have been appended to this layer already");
    if (L->prefill_unfit_head >= 0)
        return hc_fail(ctx, HC_ESHAPE, "hc_prefill_init: head %d has more refillable slots than max_k or than candidate positions",
                       L->prefill_unfit_head);
    std::vector<PreSrc> src((size_t)L->n_heads);
    for (int i = 0; i < L->n_heads; ++i) {
        if (k_src_off[i] < 0 || v_src_off[i] < 0 || (k_src_off[i] & 7) || (v_src_off[i] & 7))
            return hc_fail(ctx, HC_EINVAL, "hc_prefill_init: head %d: source offsets must be non-negative multiples of 8 elements", i);
        src[(size_t)i] = PreSrc{k_src_off[i], v_src_off[i]};
    }
    hipStream_t st = (hipStream_t)stream;
    // (pageable source: the copy has left the host buffer when the call returns)
    HC_HIP(ctx, hipMemcpyAsync(L->pre_src, src.data(), src.size() * sizeof(PreSrc), hipMemcpyHostToDevice, st));
    HC_HIP(ctx, hipStreamSynchronize(st));
    char* wb = (char*)work;
    if (L->n_sel > 0) {
        float* logits = (float*)(wb + lay.logits_off);
        float* scores = (float*)(wb + lay.scores_off);
        float* lse = (float*)(wb + lay.lse_off);
        const hc_logits_job job{L, L->sel_reps, L->n_sel, L->sel_max_len, kv_prefill, L->pre_src, q_last, logits, 0, lse, 0,
                                (float*)(wb + lay.part_off)};
        hc_status s = hc_launch_logits_lse(ctx, 1, &job, 1, st);
        if (s == HC_OK) s = hc_launch_prefill_scores(ctx, L, logits, lse, scores, pool, st);
        if (s != HC_OK) return s;
        int32_t* scratch = (int32_t*)(wb + lay.scratch_off);
        hc_monitor_call call{L, nullptr, lse, scores, topk_idx, base_idx, ring, scratch, scratch + (size_t)ctx->cfg.B * ctx->cfg.Hkv, -2};
        call.reps = L->sel_reps;
        call.outs = L->sel_outs;
        call.n_reps = call.n_outs = L->n_sel;
        call.max_nchunk = L->sel_max_nchunk;
        call.max_nk = 1;
        s = hc_launch_monitor(ctx, 1, &call, 1, st);
        if (s != HC_OK) return s;
    }
    return hc_launch_prefill_place(ctx, L, kv_prefill, kv_arena, host_tier, topk_idx, base_idx, slot_pos, ring, st);
}

// ---- re-scoring of the window's buffered queries (Algorithm 1, t mod W = 0) ----
extern "C" size_t hc_rescore_work_bytes(const hc_ctx* ctx, const hc_layer* layer)
{
    if (!ctx_ok(ctx) || !layer_ok(layer) || layer->ctx != ctx) return 0;
    return hc_rescore_plan(ctx, layer).bytes;
}

extern "C" hc_status hc_rescore_work_layout(const hc_ctx* ctx, const hc_layer* layer, int32_t* items_per_pass, size_t* logits_off,
                                            size_t* scores_off, size_t* lse_off, size_t* topk_off)
{
    if (!ctx_ok(ctx) || !layer_ok(layer) || layer->ctx != ctx) return HC_ESTATE;
    const hc_rescore_layout lay = hc_rescore_plan(ctx, layer);
    if (items_per_pass) *items_per_pass = hc_rescore_items_per_pass(ctx);
    if (logits_off) *logits_off = lay.logits_off;
    if (scores_off) *scores_off = lay.scores_off;
    if (lse_off) *lse_off = lay.lse_off;
    if (topk_off) *topk_off = lay.topk_off;
    return HC_OK;
}

static hc_status rescore_check(hc_ctx* ctx, const hc_layer* layer, const void* kv_arena, const void* q, const void* q_window,
                               const int32_t* base_idx, const int32_t* ring, const void* work, size_t work_bytes)
{
    if (!layer_ok(layer) || layer->ctx != ctx) return hc_fail(ctx, HC_ESTATE, "hc_rescore_window: layer does not belong to this context");
    if (ctx->cfg.window_mode != HC_WINDOW_RESCORED) return hc_fail(ctx, HC_ESTATE, "hc_rescore_window: the context's window_mode is not HC_WINDOW_RESCORED");
    if (!kv_arena || !q || !q_window || !base_idx || !ring || !work) return hc_fail(ctx, HC_EINVAL, "hc_rescore_window: null pointer");
    if (((uintptr_t)q | (uintptr_t)q_window) & 15) return hc_fail(ctx, HC_EINVAL, "hc_rescore_window: q and q_window must be 16-byte aligned");
    if ((uintptr_t)work & 255) return hc_fail(ctx, HC_EINVAL, "hc_rescore_window: work must be 256-byte aligned");
    if (work_bytes < hc_rescore_plan(ctx, layer).bytes)
        return hc_fail(ctx, HC_EINVAL, "hc_rescore_window: work buffer of %zu bytes, %zu needed", work_bytes, hc_rescore_plan(ctx, layer).bytes);
    return HC_OK;
}

// The passes of a test step for one or more layers (the layers of a hc_decode_step group reach the end of
// their windows together): logits and lse of up to items_per_pass buffered queries of every layer, then
// the selection passes over all (layer, query) pairs, HC_MAX_GROUP pairs to a batched call, whose last
// kernel stores each pair's overlap into its layer's ring.
struct RescoreJob {
    const hc_layer* L;
    const void* kv_arena;
    const void* q_window;
    const int32_t* base_idx;
    int32_t* ring;
    void* work;
};
static hc_status rescore_passes(hc_ctx* ctx, int n_jobs, const RescoreJob* jobs, hipStream_t st)
{
    const int W = ctx->cfg.window;
    if (W < 2) return HC_OK;
    const int per = hc_rescore_items_per_pass(ctx);
    for (int first = 0; first < W - 1; first += per) {
        const int n = std::min(per, W - 1 - first);
        {
            hc_logits_job lj[HC_MAX_GROUP];
            int n_lj = 0;
            for (int j = 0; j < n_jobs; ++j)
                if (jobs[j].L->n_reps > 0) lj[n_lj++] = hc_rescore_job(ctx, jobs[j].L, jobs[j].kv_arena, jobs[j].q_window, first, jobs[j].work);
            if (n_lj > 0) {
                const hc_status s = hc_launch_logits_lse(ctx, n_lj, lj, n, st);
                if (s != HC_OK) return s;
            }
        }
        hc_monitor_call calls[HC_MAX_GROUP];
        int n_calls = 0;
        for (int j = 0; j < n_jobs; ++j) {
            const hc_layer* L = jobs[j].L;
            if (L->n_reps == 0) continue;
            const hc_rescore_layout lay = hc_rescore_plan(ctx, L);
            char* wb = (char*)jobs[j].work;
            int32_t* scratch = (int32_t*)(wb + lay.scratch_off);
            for (int i = 0; i < n; ++i) {
                calls[n_calls++] = hc_monitor_call{L,
                                                   (const float*)(wb + lay.logits_off) + (size_t)i * lay.logits_item,
                                                   (const float*)(wb + lay.lse_off) + (size_t)i * lay.lse_item,
                                                   (float*)(wb + lay.scores_off) + (size_t)i * lay.scores_item,
                                                   (int32_t*)(wb + lay.topk_off) + (size_t)i * lay.topk_item,
                                                   const_cast<int32_t*>(jobs[j].base_idx),
                                                   jobs[j].ring,
                                                   scratch,
                                                   scratch + (size_t)ctx->cfg.B * ctx->cfg.Hkv,
                                                   first + i};
                if (n_calls == HC_MAX_GROUP || (j == n_jobs - 1 && i == n - 1)) {
                    const hc_status s = hc_launch_monitor(ctx, n_calls, calls, 0, st);
                    if (s != HC_OK) return s;
                    n_calls = 0;
                }
            }
        }
        if (n_calls > 0) {
            const hc_status s = hc_launch_monitor(ctx, n_calls, calls, 0, st);
            if (s != HC_OK) return s;
        }
    }
    return HC_OK;
}

extern "C" int32_t hc_layer_window_slot(const hc_layer* layer) { return layer_ok(layer) ? layer->window_slot : -1; }

extern "C" hc_status hc_layer_set_window_slot(hc_layer* layer, int32_t slot)
{
    if (!layer_ok(layer)) return HC_ESTATE;
    if (slot < 0 || slot >= layer->ctx->cfg.window) return hc_fail(layer->ctx, HC_EINVAL, "hc_layer_set_window_slot: slot %d outside 0..W-1", (int)slot);
    layer->window_slot = slot;
    return HC_OK;
}

extern "C" hc_status hc_rescore_window(hc_ctx* ctx, hc_layer* layer, const void* kv_arena, const void* q, void* q_window,
                                       const int32_t* base_idx, int32_t* ring, void* work, size_t work_bytes, void* stream)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    hc_status s = rescore_check(ctx, layer, kv_arena, q, q_window, base_idx, ring, work, work_bytes);
    if (s != HC_OK) return s;
    const int slot = layer->window_slot;
    layer->window_slot = (slot + 1) % ctx->cfg.window;
    hipStream_t st = (hipStream_t)stream;
    const size_t q_bytes = (size_t)ctx->cfg.B * ctx->cfg.Hq * HC_D * 2;
    const void* src = q;
    void* dst = (char*)q_window + (size_t)slot * q_bytes;
    s = hc_launch_rescore_push(ctx, 1, &src, &dst, st);
    if (s != HC_OK || slot != ctx->cfg.window - 1) return s;
    const RescoreJob job{layer, kv_arena, q_window, base_idx, ring, work};
    return rescore_passes(ctx, 1, &job, st);
}

// One decode step over a stack of layers, launched from native code so that the host keeps ahead of the
// GPU.  Layers are taken in groups: the attention of a group's layers on the main stream; then, on the
// side stream, ONE batched monitor and ONE batched gather for the whole group (seven launches per group
// instead of seven per layer: these kernels are latency-bound, so a batch costs little more GPU time than
// one layer, and the host stays ahead).  They overlap the attention of the following groups.  One event
// pair per group keeps the host cost of the cross-stream ordering small.  The attention of a layer
// waits for that layer's side work of the previous step (a refill decided at step t is used from step
// t+1; it also keeps rep_logits / lse from being overwritten while the monitor reads them).
static hc_status attn_check(hc_ctx* ctx, const hc_layer* layer, const void* kv_arena, const void* q, const float* out, const float* lse,
                            const float* rep_logits)
{
    if (!layer_ok(layer) || layer->ctx != ctx) return hc_fail(ctx, HC_ESTATE, "hc_decode_attn: layer does not belong to this context");
    if (!kv_arena || !q || !out || !lse) return hc_fail(ctx, HC_EINVAL, "hc_decode_attn: null pointer");
    if (((uintptr_t)kv_arena | (uintptr_t)q) & 15) return hc_fail(ctx, HC_EINVAL, "hc_decode_attn: kv_arena and q must be 16-byte aligned");
    if (((uintptr_t)out | (uintptr_t)lse | (uintptr_t)rep_logits) & 3) return hc_fail(ctx, HC_EINVAL, "hc_decode_attn: misaligned float pointer");
    return HC_OK;
}

extern "C" hc_status hc_decode_step(hc_ctx* ctx, const hc_layer_io* io, int32_t n_layers, int32_t layers_per_group,
                                    void* main_stream, void* side_stream)
{
    if (!ctx_ok(ctx)) return HC_ESTATE;
    if (!io || n_layers < 0 || layers_per_group < 1 || layers_per_group > HC_MAX_GROUP)
        return hc_fail(ctx, HC_EINVAL, "hc_decode_step: bad argument (layers_per_group 1..%d)", (int)HC_MAX_GROUP);
    hipStream_t ms = (hipStream_t)main_stream, ss = (hipStream_t)side_stream;
    if (side_stream != nullptr && ss == ms) return hc_fail(ctx, HC_EINVAL, "hc_decode_step: side_stream must differ from main_stream");
    // A stack that is a single group has nothing for its side work to overlap: the next step's attention waits for
    // it anyway (a refill decided at step t is used from t + 1).  Everything then runs on the main stream, which
    // saves the cross-stream events (measured with one 4K-context layer: 52 instead of 93 us per step).
    if (n_layers <= layers_per_group) ss = nullptr;
    const bool rescored = ctx->cfg.window_mode == HC_WINDOW_RESCORED;
    // Every layer's arguments are checked before anything is launched or any host-side state moves on, so that
    // a refused call leaves the whole stack as it was.
    for (int l = 0; l < n_layers; ++l) {
        const hc_layer_io& x = io[l];
        const hc_layer* L = x.layer;
        if (!layer_ok(L) || L->ctx != ctx) return hc_fail(ctx, HC_ESTATE, "hc_decode_step: layer %d does not belong to this context", l);
        for (int m = 0; m < l; ++m)
            if (io[m].layer == L) return hc_fail(ctx, HC_EINVAL, "hc_decode_step: layer %d appears twice in the stack", l);
        const bool side = L->n_reps > 0 && x.scores != nullptr;
        hc_status st = attn_check(ctx, L, x.kv_arena, x.q, x.out, x.lse, side ? x.rep_logits : nullptr);
        if (st == HC_OK && (x.k_new || x.v_new)) st = append_check(ctx, L, x.k_new, x.v_new, x.kv_arena, x.host_tier);
        if (st == HC_OK && side) {
            st = monitor_check(ctx, L, x.rep_logits, x.lse, x.scores, 0, x.topk_idx, x.base_idx, x.ring, x.inter, x.flag);
            if (st == HC_OK && rescored)
                st = rescore_check(ctx, L, x.kv_arena, x.q, x.q_window, x.base_idx, x.ring, x.rescore_work, x.rescore_work_bytes);
            if (st == HC_OK && x.host_tier && L->n_sats > 0) st = gather_check(ctx, L, x.host_tier, x.topk_idx, x.flag, x.kv_arena);
        }
        if (st != HC_OK) return st;
    }
    // The side work of a group is handed to the GPU only after the attention of the NEXT group has been: the
    // main stream then never waits for the host to get through a side chain's launches (which matters when the
    // host is slow, e.g. under a tracer), and the side chain loses nothing, since it overlaps that attention.
    struct SideWork {
        hc_monitor_call mon[HC_MAX_GROUP];
        hc_gather_call gat[HC_MAX_GROUP];
        RescoreJob test_job[HC_MAX_GROUP];
        int n_mon = 0, n_gat = 0, n_test = 0;
        bool all_filtered = true;               // every monitored layer's split pass filters its pivot logits
        hc_layer* Lg = nullptr;                 // the group's events live in its last layer
    };
    SideWork work[2];
    auto launch_side = [&](SideWork& w) -> hc_status {
        if (w.n_mon == 0) return HC_OK;
        hipStream_t run = ss ? ss : ms;
        if (ss) HC_HIP(ctx, hipStreamWaitEvent(ss, w.Lg->ev_attn, 0));
        hc_status st = HC_OK;
        if (w.n_test > 0) st = rescore_passes(ctx, w.n_test, w.test_job, run);       // test step of a re-scored window: the earlier queries first
        ctx->side_pad_now = ss != nullptr && w.all_filtered;
        if (st == HC_OK) st = hc_launch_monitor(ctx, w.n_mon, w.mon, 0, run);
        if (st == HC_OK && w.n_gat > 0) st = hc_launch_gather(ctx, w.n_gat, w.gat, run);
        ctx->side_pad_now = false;
        if (ss) {
            // recorded even after a failed launch, so that no later call waits on a stale event
            const hipError_t e = hipEventRecord(w.Lg->ev_side, ss);
            for (int i = 0; i < w.n_mon; ++i) const_cast<hc_layer*>(w.mon[i].L)->pending_ev = w.Lg->ev_side;
            if (st == HC_OK) HC_HIP(ctx, e);
        }
        w.n_mon = 0;
        return st;
    };
    hipEvent_t last_waited = nullptr;
    int cur = 0;
    hc_status result = HC_OK;
    for (int g0 = 0; g0 < n_layers && result == HC_OK; g0 += layers_per_group) {
        const int g1 = std::min(n_layers, g0 + layers_per_group);
        SideWork& w = work[cur];
        w.n_mon = w.n_gat = w.n_test = 0;
        w.all_filtered = true;
        const void* push_src[HC_MAX_GROUP];
        void* push_dst[HC_MAX_GROUP];
        hc_layer* push_layer[HC_MAX_GROUP];
        int n_push = 0;
        // the tokens of the group's layers enter their caches with one launch, ahead of the group's attention
        hc_append_call app[HC_MAX_GROUP];
        int n_app = 0;
        for (int l = g0; l < g1; ++l) {
            const hc_layer_io& x = io[l];
            hc_layer* L = x.layer;
            if (L->pending_ev) {
                if (L->pending_ev != last_waited) {
                    const hipError_t e = hipStreamWaitEvent(ms, L->pending_ev, 0);
                    if (e != hipSuccess) result = hc_fail(ctx, HC_EHIP, "hc_decode_step: hipStreamWaitEvent: %s", hipGetErrorString(e));
                }
                last_waited = L->pending_ev;
                L->pending_ev = nullptr;
            }
            if (x.k_new || x.v_new)
                app[n_app++] = hc_append_call{L, x.k_new, x.v_new, const_cast<void*>(x.kv_arena), const_cast<void*>(x.host_tier)};
        }
        if (result == HC_OK && n_app > 0) {
            result = hc_launch_append(ctx, n_app, app, ms);
            for (int i = 0; i < n_app && result == HC_OK; ++i) result = append_done(ctx, const_cast<hc_layer*>(app[i].L), ms);
        }
        for (int l = g0; l < g1 && result == HC_OK; ++l) {
            const hc_layer_io& x = io[l];
            hc_layer* L = x.layer;
            const bool side = L->n_reps > 0 && x.scores != nullptr;
            if (side) {
                w.mon[w.n_mon] = hc_monitor_call{L, x.rep_logits, x.lse, x.scores, x.topk_idx, x.base_idx, x.ring, x.inter, x.flag};
                w.mon[w.n_mon++].arena = x.kv_arena;
                L->last_arena = x.kv_arena;
                w.all_filtered = w.all_filtered && hc_layer_filtered(ctx, L);
                if (rescored) {
                    push_src[n_push] = x.q;
                    push_layer[n_push] = L;
                    push_dst[n_push++] = (char*)x.q_window + (size_t)L->window_slot * ctx->cfg.B * ctx->cfg.Hq * HC_D * 2;
                    if (L->window_slot == ctx->cfg.window - 1)
                        w.test_job[w.n_test++] = RescoreJob{L, x.kv_arena, x.q_window, x.base_idx, x.ring, x.rescore_work};
                }
                if (x.host_tier && L->n_sats > 0)
                    w.gat[w.n_gat++] = hc_gather_call{L, x.host_tier, x.topk_idx, x.flag, const_cast<void*>(x.kv_arena), x.slot_pos};
            }
            result = hc_launch_attn(ctx, L, x.kv_arena, x.q, x.out, x.lse, side ? x.rep_logits : nullptr, ms);
        }
        // The queries go into the window buffers on the main stream: the caller may overwrite q as soon
        // as this call returns, in main-stream order, while the side stream may still be behind.  A layer's
        // count of steps inside its window moves on once its query is in the buffer.
        if (result == HC_OK && n_push > 0) {
            result = hc_launch_rescore_push(ctx, n_push, push_src, push_dst, ms);
            if (result == HC_OK)
                for (int i = 0; i < n_push; ++i) push_layer[i]->window_slot = (push_layer[i]->window_slot + 1) % ctx->cfg.window;
        }
        if (result != HC_OK) w.n_mon = 0;              // this group's side work is dropped; the previous group's still goes out
        if (w.n_mon > 0) {
            w.Lg = io[g1 - 1].layer;
            if (ss) {
                const hipError_t e = hipEventRecord(w.Lg->ev_attn, ms);
                if (e != hipSuccess) { result = hc_fail(ctx, HC_EHIP, "hc_decode_step: hipEventRecord: %s", hipGetErrorString(e)); w.n_mon = 0; }
            }
        }
        const hc_status sp = launch_side(work[cur ^ 1]);
        if (result == HC_OK) result = sp;
        cur ^= 1;
    }
    const hc_status sl = launch_side(work[cur ^ 1]);
    if (result == HC_OK) result = sl;
    return result;
}
