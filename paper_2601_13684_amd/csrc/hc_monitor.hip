// hc_monitor.hip -- the pivot heads' drift monitor (Sec. 4.3, Eq. 9-10; Algorithm 1 stage 3):
// GQA-aggregated score (App. C.1), TopIndices_k for every needed set size, overlap with the
// baseline set, windowed-median retrieval signal, baseline update.
//
// Selection is an exact 3-digit radix select (11 + 11 + 10 bits) on order-preserving 32-bit keys of
// the fp32 scores, run by many workgroups per pivot because the score array (up to ~1 MB) is far
// too long for one.  Ties at the threshold key are resolved by position: the equal-keyed candidates
// with the lowest indices are taken, which makes the result the unique first-k set under
// (score descending, index ascending).  The lists are emitted in ascending index order by an
// ordered compaction (per-chunk counts, then prefix sums).
//
// Kernels, all on the caller's stream:
//   mon_prep        clear histograms, selection state, accumulators and the baseline bitmap
//   mon_score_hist  score + first-digit histogram; scatter the baseline list into the bitmap
//   mon_hist<2>     find the first digit of every set size; histogram of the second digit
//   mon_hist<3>     find the second digit; histogram of the third digit
//   mon_count       find the threshold key; per-chunk counts of greater / equal keys
//   mon_write       ordered compaction into topk_idx; |T ∩ baseline| through the bitmap; the last
//                   workgroup of a pivot's monitored list takes the trigger decision (exact integer
//                   form of Eq. 10), writes inter / flag / ring and, on a trigger, the new baseline.
#include "hc_internal.h"

namespace {

constexpr int BLK = 256;
constexpr int PER_THREAD = HC_SEL_CHUNK / BLK;   // 16

__device__ __forceinline__ uint32_t score_key(float s)
{
    uint32_t u = __float_as_uint(s);
    if (s != s) return 0u;                    // NaN ranks below everything
    if (u == 0x80000000u) u = 0u;             // -0 and +0 are the same score
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

struct RepWs {
    uint32_t* h1;     // [HC_RADIX_BINS]
    uint32_t* h2;     // [HC_MAX_K_PER_REP][HC_RADIX_BINS]
    uint32_t* h3;     // [HC_MAX_K_PER_REP][HC_RADIX_BINS]
    uint32_t* sel;    // [HC_MAX_K_PER_REP][4]: digit-1 prefix / remaining, then 22-bit prefix / remaining, then tau / need
    uint32_t* misc;   // [4]: intersection accumulator, ticket
    uint32_t* cnt;    // [HC_MAX_K_PER_REP][max_chunks][2]
    uint32_t* bitmap; // [max_ctx/32]
};

struct Ws {
    uint32_t *hist, *sel, *misc, *cnt, *bitmap;
    int max_chunks, max_ctx;
    __device__ RepWs rep(int r) const
    {
        RepWs w;
        uint32_t* h = hist + (size_t)r * (1 + 2 * HC_MAX_K_PER_REP) * HC_RADIX_BINS;
        w.h1 = h;
        w.h2 = h + HC_RADIX_BINS;
        w.h3 = h + (size_t)(1 + HC_MAX_K_PER_REP) * HC_RADIX_BINS;
        w.sel = sel + (size_t)r * HC_MAX_K_PER_REP * 4;
        w.misc = misc + (size_t)r * 4;
        w.cnt = cnt + (size_t)r * HC_MAX_K_PER_REP * max_chunks * 2;
        w.bitmap = bitmap + (size_t)r * (max_ctx / 32);
        return w;
    }
};

// Exclusive prefix sum over the 256 threads of the workgroup; also returns the total.
__device__ __forceinline__ uint32_t block_exscan(uint32_t v, uint32_t* sm /*[5]*/, uint32_t& total)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    __syncthreads();
    if (lane == 63) sm[w] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t x = sm[i];
        if (i < w) base += x;
        tot += x;
    }
    total = tot;
    return base + inc - v;
}

// In a histogram of `nbins` (<= 2048) digit counts, walking from the highest digit down, find the
// digit in which the k-th largest element falls and how many of that digit's elements are still
// needed.  All threads return the same result.
__device__ __forceinline__ void find_digit(const uint32_t* __restrict__ hist, int nbins, uint32_t k,
                                           uint32_t* sm /*[8]*/, uint32_t& digit, uint32_t& remaining)
{
    // thread t owns the 8 digits nbins-1-8t ... nbins-8-8t (descending)
    uint32_t h[8];
    uint32_t local = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int b = nbins - 1 - (threadIdx.x * 8 + i);
        h[i] = (b >= 0) ? hist[b] : 0u;
        local += h[i];
    }
    uint32_t total;
    uint32_t above = block_exscan(local, sm, total);     // elements in higher digits than mine
    __syncthreads();
    if (above < k && k <= above + local) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (above < k && k <= above + h[i]) {
                sm[5] = (uint32_t)(nbins - 1 - (threadIdx.x * 8 + i));
                sm[6] = k - above;
            }
            above += h[i];
        }
    }
    __syncthreads();
    digit = sm[5];
    remaining = sm[6];
    __syncthreads();
}

__global__ __launch_bounds__(BLK) void mon_prep(Ws ws, const RepDev* __restrict__ reps)
{
    const int rep = blockIdx.y;
    const RepWs w = ws.rep(rep);
    const size_t hist_words = (size_t)(1 + 2 * HC_MAX_K_PER_REP) * HC_RADIX_BINS;
    const size_t bm_words = (size_t)(reps[rep].hi + 31) / 32;
    const size_t stride = (size_t)gridDim.x * BLK;
    for (size_t i = (size_t)blockIdx.x * BLK + threadIdx.x; i < hist_words; i += stride) w.h1[i] = 0u;
    for (size_t i = (size_t)blockIdx.x * BLK + threadIdx.x; i < bm_words; i += stride) w.bitmap[i] = 0u;
    if (blockIdx.x == 0) {
        if (threadIdx.x < HC_MAX_K_PER_REP * 4) w.sel[threadIdx.x] = 0u;
        if (threadIdx.x < 4) w.misc[threadIdx.x] = 0u;
    }
}

__global__ __launch_bounds__(BLK) void mon_score_hist(Ws ws, const RepDev* __restrict__ reps,
                                                      const float* __restrict__ rep_logits,
                                                      const float* __restrict__ lse, float* __restrict__ scores,
                                                      int scores_given, int G, int agg,
                                                      const int32_t* __restrict__ base_idx, int max_k)
{
    __shared__ uint32_t sh[HC_RADIX_BINS];
    const int rep = blockIdx.y;
    const RepDev rd = reps[rep];
    if ((int)blockIdx.x >= rd.nchunk) return;
    const RepWs w = ws.rep(rep);
    for (int i = threadIdx.x; i < HC_RADIX_BINS; i += BLK) sh[i] = 0u;

    // baseline list -> bitmap (each workgroup takes a slice of the list)
    const int32_t* base = base_idx + (size_t)rd.bh * max_k;
    for (int i = blockIdx.x * BLK + threadIdx.x; i < rd.k[0]; i += rd.nchunk * BLK) {
        const int j = base[i];
        if (j >= rd.lo && j < rd.hi) atomicOr(&w.bitmap[j >> 5], 1u << (j & 31));
    }
    __syncthreads();

    float* srow = scores + (size_t)rep * ws.max_ctx;
    const float* lrow = rep_logits ? rep_logits + (size_t)rep * G * ws.max_ctx : nullptr;
    float l[8];
    if (!scores_given && agg == HC_AGG_PROB)
        for (int g = 0; g < G; ++g) l[g] = lse[(size_t)rd.bh * G + g];
    const float invG = 1.0f / (float)G;
    const int first = rd.lo + blockIdx.x * HC_SEL_CHUNK;
    for (int i = 0; i < PER_THREAD; ++i) {
        const int j = first + i * BLK + threadIdx.x;
        if (j >= rd.hi) break;
        float s;
        if (scores_given) {
            s = srow[j];
        } else {
            float a = 0.f;
            if (agg == HC_AGG_PROB) {
                for (int g = 0; g < G; ++g) a += expf(lrow[(size_t)g * ws.max_ctx + j] - l[g]);
            } else if (G == 4) {
                a = (lrow[j] + lrow[(size_t)ws.max_ctx + j]) + (lrow[(size_t)2 * ws.max_ctx + j] + lrow[(size_t)3 * ws.max_ctx + j]);
            } else {
                for (int g = 0; g < G; ++g) a += lrow[(size_t)g * ws.max_ctx + j];
            }
            s = a * invG;
            srow[j] = s;
        }
        atomicAdd(&sh[score_key(s) >> 21], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < HC_RADIX_BINS; i += BLK)
        if (sh[i]) atomicAdd(&w.h1[i], sh[i]);
}

// PASS 2: digit two (bits 20..10) among keys whose first digit matches; PASS 3: digit three (bits 9..0)
// among keys whose upper 22 bits match.
template <int PASS>
__global__ __launch_bounds__(BLK) void mon_hist(Ws ws, const RepDev* __restrict__ reps, const float* __restrict__ scores)
{
    __shared__ uint32_t sh[HC_RADIX_BINS];
    __shared__ uint32_t sm[8];
    const int rep = blockIdx.y / HC_MAX_K_PER_REP, ks = blockIdx.y % HC_MAX_K_PER_REP;
    const RepDev rd = reps[rep];
    if (ks >= rd.nk || (int)blockIdx.x >= rd.nchunk) return;
    const RepWs w = ws.rep(rep);
    for (int i = threadIdx.x; i < HC_RADIX_BINS; i += BLK) sh[i] = 0u;

    uint32_t prefix, remaining;
    if (PASS == 2) {
        find_digit(w.h1, HC_RADIX_BINS, (uint32_t)rd.k[ks], sm, prefix, remaining);
    } else {
        uint32_t d2;
        find_digit(w.h2 + (size_t)ks * HC_RADIX_BINS, HC_RADIX_BINS, w.sel[ks * 4 + 1], sm, d2, remaining);
        prefix = (w.sel[ks * 4 + 0] << 11) | d2;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {   // state for the next pass (same value from every workgroup)
        if (PASS == 2) {
            w.sel[ks * 4 + 0] = prefix;
            w.sel[ks * 4 + 1] = remaining;
        } else {
            w.sel[ks * 4 + 2] = prefix;
            w.sel[ks * 4 + 3] = remaining;
        }
    }
    const float* srow = scores + (size_t)rep * ws.max_ctx;
    const int first = rd.lo + blockIdx.x * HC_SEL_CHUNK;
    for (int i = 0; i < PER_THREAD; ++i) {
        const int j = first + i * BLK + threadIdx.x;
        if (j >= rd.hi) break;
        const uint32_t key = score_key(srow[j]);
        if (PASS == 2) {
            if ((key >> 21) == prefix) atomicAdd(&sh[(key >> 10) & 0x7ffu], 1u);
        } else {
            if ((key >> 10) == prefix) atomicAdd(&sh[key & 0x3ffu], 1u);
        }
    }
    __syncthreads();
    uint32_t* gh = (PASS == 2 ? w.h2 : w.h3) + (size_t)ks * HC_RADIX_BINS;
    for (int i = threadIdx.x; i < HC_RADIX_BINS; i += BLK)
        if (sh[i]) atomicAdd(&gh[i], sh[i]);
}

__global__ __launch_bounds__(BLK) void mon_count(Ws ws, const RepDev* __restrict__ reps, const float* __restrict__ scores)
{
    __shared__ uint32_t sm[8];
    __shared__ uint32_t red[2][4];
    const int rep = blockIdx.y / HC_MAX_K_PER_REP, ks = blockIdx.y % HC_MAX_K_PER_REP;
    const RepDev rd = reps[rep];
    if (ks >= rd.nk || (int)blockIdx.x >= rd.nchunk) return;
    const RepWs w = ws.rep(rep);
    uint32_t d3, need;
    find_digit(w.h3 + (size_t)ks * HC_RADIX_BINS, 1024, w.sel[ks * 4 + 3], sm, d3, need);
    const uint32_t tau = (w.sel[ks * 4 + 2] << 10) | d3;
    const float* srow = scores + (size_t)rep * ws.max_ctx;
    const int first = rd.lo + blockIdx.x * HC_SEL_CHUNK;
    uint32_t gt = 0, eq = 0;
    for (int i = 0; i < PER_THREAD; ++i) {
        const int j = first + i * BLK + threadIdx.x;
        if (j >= rd.hi) break;
        const uint32_t key = score_key(srow[j]);
        gt += key > tau;
        eq += key == tau;
    }
    for (int o = 32; o > 0; o >>= 1) {
        gt += __shfl_xor(gt, o);
        eq += __shfl_xor(eq, o);
    }
    if ((threadIdx.x & 63) == 0) {
        red[0][threadIdx.x >> 6] = gt;
        red[1][threadIdx.x >> 6] = eq;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t* c = w.cnt + ((size_t)ks * ws.max_chunks + blockIdx.x) * 2;
        c[0] = red[0][0] + red[0][1] + red[0][2] + red[0][3];
        c[1] = red[1][0] + red[1][1] + red[1][2] + red[1][3];
    }
    // The first workgroup leaves tau / need for mon_write.  It must not overwrite sel[2..3] before
    // every other workgroup of this launch has read them, so the pair goes to the (now dead) first
    // two words, which this kernel does not read.
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        w.sel[ks * 4 + 0] = tau;
        w.sel[ks * 4 + 1] = need;
    }
}

struct DriftCfg {
    int window, metric, tau_num, tau_den, max_k;
};

__global__ __launch_bounds__(BLK) void mon_write(Ws ws, const RepDev* __restrict__ reps, const OutDev* __restrict__ outs,
                                                 const float* __restrict__ scores, int32_t* __restrict__ topk_idx,
                                                 int32_t* __restrict__ base_idx, int32_t* __restrict__ ring,
                                                 int32_t* __restrict__ inter_out, int32_t* __restrict__ flag_out,
                                                 DriftCfg cfg)
{
    __shared__ uint32_t sm[8];
    __shared__ uint32_t sm_off[2];
    __shared__ uint32_t sm_last;
    const OutDev od = outs[blockIdx.y];
    const RepDev rd = reps[od.rep];
    const int chunk = blockIdx.x;
    if (chunk >= rd.nchunk) return;
    const RepWs w = ws.rep(od.rep);
    const int ks = od.kslot;
    const uint32_t tau = w.sel[ks * 4 + 0], need = w.sel[ks * 4 + 1];
    const int k = rd.k[ks];

    // Prefix over the chunks before mine: equal-keyed candidates seen, and list entries emitted.
    // A chunk emits all its greater keys plus as many equal keys as are still needed.
    {
        const uint32_t* cnt = w.cnt + (size_t)ks * ws.max_chunks * 2;
        // equal-key prefix is sequential in nature; chunks are few (<= max_ctx/4096), so one thread walks them
        if (threadIdx.x == 0) {
            uint32_t eq_before = 0, emitted = 0;
            for (int c = 0; c < chunk; ++c) {
                const uint32_t g = cnt[c * 2], e = cnt[c * 2 + 1];
                const uint32_t left = need > eq_before ? need - eq_before : 0u;
                emitted += g + (e < left ? e : left);
                eq_before += e;
            }
            sm_off[0] = eq_before;
            sm_off[1] = emitted;
        }
        __syncthreads();
    }
    const uint32_t eq_before_chunk = sm_off[0];
    const uint32_t out_base = sm_off[1];

    // each thread owns 16 consecutive candidates so that the compaction keeps index order
    const float* srow = scores + (size_t)od.rep * ws.max_ctx;
    const int first = rd.lo + chunk * HC_SEL_CHUNK + threadIdx.x * PER_THREAD;
    uint32_t keys[PER_THREAD];
    uint32_t my_eq = 0;
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
        const int j = first + i;
        keys[i] = (j < rd.hi) ? score_key(srow[j]) : 0u;
        if (j < rd.hi && keys[i] == tau) ++my_eq;
    }
    uint32_t tot;
    uint32_t eq_rank = eq_before_chunk + block_exscan(my_eq, sm, tot);
    __syncthreads();
    uint32_t selmask = 0, my_sel = 0;
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
        const int j = first + i;
        if (j >= rd.hi) break;
        bool s = keys[i] > tau;
        if (keys[i] == tau) {
            s = eq_rank < need;
            ++eq_rank;
        }
        if (s) {
            selmask |= 1u << i;
            ++my_sel;
        }
    }
    uint32_t pos = out_base + block_exscan(my_sel, sm, tot);
    int32_t* dst = topk_idx + (size_t)od.row * cfg.max_k;
    uint32_t hits = 0;
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
        if (selmask & (1u << i)) {
            const int j = first + i;
            if (pos < (uint32_t)k) dst[pos] = j;     // pos < k always holds; the guard keeps a corrupt state in bounds
            ++pos;
            if (od.is_mon) hits += (w.bitmap[j >> 5] >> (j & 31)) & 1u;
        }
    }
    if (!od.is_mon) return;

    // ---- monitored list only: intersection size, then the decision by the last workgroup ----
    for (int o = 32; o > 0; o >>= 1) hits += __shfl_xor(hits, o);
    if ((threadIdx.x & 63) == 0 && hits) atomicAdd(&w.misc[0], hits);
    __threadfence();          // my list entries and my hits are visible before my ticket
    __syncthreads();
    if (threadIdx.x == 0) sm_last = (atomicAdd(&w.misc[1], 1u) == (uint32_t)rd.nchunk - 1u);
    __syncthreads();
    if (!sm_last) return;
    __threadfence();          // see what the other workgroups wrote
    if (threadIdx.x == 0) {
        const int32_t inter = (int32_t)__hip_atomic_load(&w.misc[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int32_t* rg = ring + (size_t)rd.bh * (cfg.window + 1);
        int n = rg[0];
        if (n < 0 || n > cfg.window) n = 0;
        if (n == cfg.window) {                       // sliding window: drop the oldest value
            for (int i = 1; i < cfg.window; ++i) rg[i] = rg[i + 1];
            n = cfg.window - 1;
        }
        rg[1 + n] = inter;
        ++n;
        int trig = 0;
        if (n == cfg.window) {
            int32_t tmp[HC_MAX_WINDOW];
            for (int i = 0; i < n; ++i) tmp[i] = rg[1 + i];
            for (int i = 1; i < n; ++i) {            // insertion sort, W <= 64
                const int32_t v = tmp[i];
                int p = i - 1;
                while (p >= 0 && tmp[p] > v) {
                    tmp[p + 1] = tmp[p];
                    --p;
                }
                tmp[p + 1] = v;
            }
            const long long med = tmp[(n - 1) / 2];  // lower median
            const long long kk = k;
            if (cfg.metric == HC_METRIC_OVERLAP)
                trig = med * cfg.tau_den < (long long)cfg.tau_num * kk;                     // med/k < tau
            else
                trig = med * cfg.tau_den < (long long)cfg.tau_num * (2 * kk - med);         // med/(2k-med) < tau
        }
        if (trig) n = 0;                             // the window restarts after a retrieval
        rg[0] = n;
        inter_out[rd.bh] = inter;
        flag_out[rd.bh] = trig;
        sm[7] = (uint32_t)trig;
    }
    __syncthreads();
    if (sm[7]) {                                     // K_base <- K_t
        int32_t* base = base_idx + (size_t)rd.bh * cfg.max_k;
        for (int i = threadIdx.x; i < k; i += BLK)
            base[i] = __hip_atomic_load(&dst[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

}   // namespace

hc_status hc_launch_monitor(hc_ctx* ctx, const hc_layer* L, const float* rep_logits, const float* lse, float* scores,
                            int scores_given, int32_t* topk_idx, int32_t* base_idx, int32_t* ring, int32_t* inter,
                            int32_t* flag, hipStream_t st)
{
    Ws ws{ctx->hist, ctx->sel, ctx->misc, ctx->cnt, ctx->bitmap, ctx->max_chunks, ctx->cfg.max_ctx};
    const hc_config& c = ctx->cfg;
    const dim3 blk(BLK);
    mon_prep<<<dim3(16, L->n_reps), blk, 0, st>>>(ws, L->reps);
    HC_HIP(ctx, hipGetLastError());
    mon_score_hist<<<dim3(L->max_nchunk, L->n_reps), blk, 0, st>>>(ws, L->reps, rep_logits, lse, scores, scores_given,
                                                                   ctx->G, c.agg, base_idx, c.max_k);
    HC_HIP(ctx, hipGetLastError());
    const dim3 gk(L->max_nchunk, L->n_reps * HC_MAX_K_PER_REP);
    mon_hist<2><<<gk, blk, 0, st>>>(ws, L->reps, scores);
    HC_HIP(ctx, hipGetLastError());
    mon_hist<3><<<gk, blk, 0, st>>>(ws, L->reps, scores);
    HC_HIP(ctx, hipGetLastError());
    mon_count<<<gk, blk, 0, st>>>(ws, L->reps, scores);
    HC_HIP(ctx, hipGetLastError());
    DriftCfg dc{c.window, c.metric, c.tau_num, c.tau_den, c.max_k};
    mon_write<<<dim3(L->max_nchunk, L->n_outs), blk, 0, st>>>(ws, L->reps, L->outs, scores, topk_idx, base_idx, ring,
                                                             inter, flag, dc);
    HC_HIP(ctx, hipGetLastError());
    return HC_OK;
}
