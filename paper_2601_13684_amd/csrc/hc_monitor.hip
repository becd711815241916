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
// The work is latency-bound, not bandwidth-bound (a few MB, L2-resident), so every kernel is shaped to
// have few dependent memory round trips: four candidates per thread fetched with one 16-byte load, all set
// sizes of a pivot handled in the same pass over the scores, no local arrays (no scratch memory) and no
// device-wide fences (the decision has a kernel of its own instead).  Workgroups are 256 threads with few
// registers so that they can share compute units with the attention pass of the next layer when the
// caller runs the monitor on a side stream.
//
// Kernels, all on the caller's stream:
//   (mon_prep       clear the digit histograms and the baseline bitmap: only after a failed call; normally
//                   they are left clear by the previous call's last kernel)
//   mon_score_hist  score + first-digit histogram; scatter the baseline list into the bitmap
//   mon_hist<2>     find the first digit of every set size; histograms of the second digit
//   mon_hist<3>     find the second digit; histograms of the third digit
//   mon_count       find the threshold key; per-chunk counts of greater / equal keys
//   mon_write       ordered compaction into topk_idx; |T ∩ baseline| through the bitmap
//   mon_decide      window update and trigger decision (exact integer form of Eq. 10): writes inter, flag,
//                   ring and, on a trigger, the new baseline; clears histograms and bitmap for the next call
#include "hc_internal.h"

namespace {

constexpr int BLK = 256;     // small workgroups: they fit beside the attention pass's waves on a compute unit
constexpr int PER_THREAD = HC_SEL_CHUNK / BLK;   // 4 consecutive candidates per thread
static_assert(PER_THREAD == 4, "one 16-byte load per thread");
constexpr int NWAVE = BLK / 64;
static_assert(NWAVE == 4, "reductions below add four wave sums");

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
    uint32_t *hist, *sel, *misc, *cnt, *bitmap, *hits;
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

// One layer of a batched call: its workspace copy, its plan and the caller's buffers.  A launch handles
// up to HC_MAX_GROUP layers (blockIdx.z picks the layer), so that a group of layers costs the launches
// and the launch latencies of one.
struct MonItem {
    Ws ws;
    const RepDev* reps;
    const OutDev* outs;
    const float* rep_logits;
    const float* lse;
    float* scores;
    int32_t* topk_idx;
    int32_t* base_idx;
    int32_t* ring;
    int32_t* inter;
    int32_t* flag;
    int n_reps, n_outs;
    int store_slot;
    // A layer whose split pass filters the pivot logits: the selection passes run over the kept rows only
    // (reps = the pivots as seen over those rows, pos_map = their positions), and a second, dense chain of the
    // same passes stands by for the pivots whose check failed (need[rep] != 0).
    int need_sense;               // -1: unconditional; 0: run where need[rep] == 0; 1: run where need[rep] != 0
    const int32_t* need_r;        // [n_reps], read by every pass
    int32_t* need_w;              // the same table, written by the first pass and the check
    const RepDev* real_reps;      // the pivots by position (candidate range, table row); == reps unless filtered
    const int32_t* pos_map;       // [n_reps][max_ctx] position of every kept row, or nullptr: a row is its position
    int32_t* dense_pos;           // the same table, written by the first filtered pass
    const HeadDev* heads;         // filtered first pass: where a pivot's segments are ...
    const SegDev* segs;           // ... which rows of the pivot's block they begin at ...
    const int32_t* seg_cnt;       // ... and how many rows each of them kept
    const int32_t* surv_pos;      // [n_reps][max_ctx] positions of the kept rows, by segment
    RepDev* vreps;                // written by the first filtered pass
    RepFilter* filt;              // checked (this step's) and set (the next step's) when not nullptr
    uint32_t* counts;             // [n_reps][4] or nullptr
    int cap_rows;                 // filtered: more kept rows than this (or fewer than the largest list) go to the dense chain
    float margin;                 // filter for the next step: cut = smallest list threshold / margin
};
struct MonBatch {
    MonItem it[HC_MAX_GROUP];
};

__device__ __forceinline__ bool mon_skip(const MonItem& it, int rep)
{
    return it.need_sense >= 0 && ((it.need_r[rep] != 0) != (it.need_sense != 0));
}

__device__ __forceinline__ float key_score(uint32_t key)      // inverse of score_key
{
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

__device__ __forceinline__ uint32_t wave_exscan(uint32_t v, uint32_t& total)
{
    const int lane = threadIdx.x & 63;
    uint32_t inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    total = __shfl(inc, 63);
    return inc - v;
}

// In a histogram of nbins (<= 2048) digit counts, walking from the highest digit down, find the digit
// in which the k-th largest element falls and how many of that digit's elements are still needed.
// Done by ONE wave (lane l owns 32 consecutive digits); result valid in all its lanes.
template <int nbins>
__device__ __forceinline__ void find_digit_wave(const uint32_t* __restrict__ hist, uint32_t k, uint32_t& digit,
                                                uint32_t& remaining)
{
    const int lane = threadIdx.x & 63;
    constexpr int per = nbins / 64;               // 32 or 16
    // lane l owns digits nbins-1-l*per ... nbins-(l+1)*per (descending)
    uint32_t local = 0;
    const uint4* h4 = reinterpret_cast<const uint4*>(hist + (nbins - (lane + 1) * per));
    uint4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if (i < per / 4) {
            v[i] = h4[i];
            local += v[i].x + v[i].y + v[i].z + v[i].w;
        }
    uint32_t tot;
    uint32_t above = wave_exscan(local, tot);      // elements in higher digits than this lane's
    const bool mine = above < k && k <= above + local;
    uint32_t d = 0, rem = 0;
    if (mine) {
        // walk this lane's digits from the highest (last word of its span) down
#pragma unroll
        for (int i = per - 1; i >= 0; --i) {
            const uint4 q = v[i >> 2];
            const uint32_t c = (i & 3) == 0 ? q.x : (i & 3) == 1 ? q.y : (i & 3) == 2 ? q.z : q.w;
            if (above < k && k <= above + c) {
                d = (uint32_t)(nbins - (lane + 1) * per + i);
                rem = k - above;
            }
            above += c;
        }
    }
    const uint64_t who = __builtin_amdgcn_ballot_w64(mine);
    const int src = who ? __builtin_ctzll(who) : 0;
    digit = __shfl(d, src);
    remaining = __shfl(rem, src);
}

__global__ __launch_bounds__(256) void mon_prep(Ws ws, int max_ctx)
{
    const RepWs w = ws.rep(blockIdx.y);
    const size_t hist_words = (size_t)(1 + 2 * HC_MAX_K_PER_REP) * HC_RADIX_BINS;
    const size_t bm_words = (size_t)max_ctx / 32;
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < hist_words; i += stride) w.h1[i] = 0u;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < bm_words; i += stride) w.bitmap[i] = 0u;
}

// Score of candidate j from the G scaled logits of its row (rep_logits is [ctx][G] per pivot).
template <int G>
__device__ __forceinline__ float score_of(const float* __restrict__ lrow, int j, const float (&lse)[G], int agg)
{
    float l[G];
    if (G == 1) {
        l[0] = lrow[j];
    } else if (G == 2) {
        const float2 v = reinterpret_cast<const float2*>(lrow)[j];
        l[0] = v.x; l[1] = v.y;
    } else {
#pragma unroll
        for (int q = 0; q < G / 4; ++q) {
            const float4 v = reinterpret_cast<const float4*>(lrow)[(size_t)j * (G / 4) + q];
            l[4 * q] = v.x; l[4 * q + 1] = v.y; l[4 * q + 2] = v.z; l[4 * q + 3] = v.w;
        }
    }
    float a;
    if (agg == HC_AGG_PROB) {
        a = 0.f;
#pragma unroll
        for (int g = 0; g < G; ++g) a += expf(l[g] - lse[g]);
    } else if (G == 4) {
        a = (l[0] + l[1]) + (l[2] + l[3]);
    } else {
        a = 0.f;
#pragma unroll
        for (int g = 0; g < G; ++g) a += l[g];
    }
    return a * (1.0f / (float)G);
}

// A workgroup of the selection passes takes `span` consecutive chunks of HC_SEL_CHUNK candidates: 1 when a
// single layer is handled (many small workgroups: latency), more when a batch of layers is (the histograms
// in LDS are cleared and flushed once per workgroup, so fewer, longer workgroups do far less work in total
// and a batch fits a small part of the GPU).
template <int G>
__global__ __launch_bounds__(BLK) void mon_score_hist(MonBatch B, int scores_given, int agg, int max_k, int span)
{
    __shared__ uint32_t sh[HC_RADIX_BINS];
    const MonItem& it = B.it[blockIdx.z];
    const int rep = blockIdx.y;
    if (rep >= it.n_reps || mon_skip(it, rep)) return;
    const Ws ws = it.ws;
    const RepDev* __restrict__ reps = it.reps;
    const float* __restrict__ rep_logits = it.rep_logits;
    const float* __restrict__ lse = it.lse;
    float* __restrict__ scores = it.scores;
    const int32_t* __restrict__ base_idx = it.base_idx;
    const RepDev rd = reps[rep];
    const int c0 = blockIdx.x * span, c1 = min(c0 + span, rd.nchunk);
    if (c0 >= rd.nchunk) return;
    const RepWs w = ws.rep(rep);
    for (int i = threadIdx.x; i < HC_RADIX_BINS; i += BLK) sh[i] = 0u;

    // baseline list -> bitmap (each workgroup takes a slice of the list)
    const int32_t* base = base_idx + (size_t)rd.bh * max_k;
    const int nblk = (rd.nchunk + span - 1) / span;
    for (int i = blockIdx.x * BLK + threadIdx.x; i < rd.k[0]; i += nblk * BLK) {
        const int j = base[i];
        if (j >= rd.lo && j < rd.hi) atomicOr(&w.bitmap[j >> 5], 1u << (j & 31));
    }
    __syncthreads();

    float* srow = scores + (size_t)rep * ws.max_ctx;
    const float* lrow = rep_logits ? rep_logits + (size_t)rep * G * ws.max_ctx : nullptr;
    float l[G];
#pragma unroll
    for (int g = 0; g < G; ++g) l[g] = (!scores_given && agg == HC_AGG_PROB) ? lse[(size_t)rd.bh * G + g] : 0.f;
    for (int ch = c0; ch < c1; ++ch) {
        const int first = rd.lo + ch * HC_SEL_CHUNK;
        float s[PER_THREAD];
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {       // candidate first + i*BLK + t: coalesced, loads independent
            const int j = first + i * BLK + threadIdx.x;
            s[i] = 0.f;
            if (j < rd.hi) s[i] = scores_given ? srow[j] : score_of<G>(lrow, j, l, agg);
        }
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int j = first + i * BLK + threadIdx.x;
            if (j < rd.hi) {
                if (!scores_given) srow[j] = s[i];
                atomicAdd(&sh[score_key(s[i]) >> 21], 1u);
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < HC_RADIX_BINS; i += BLK)
        if (sh[i]) atomicAdd(&w.h1[i], sh[i]);
}

// The four candidates of a thread: positions first4 .. first4+3 (first4 a multiple of 4, so one
// 16-byte load), of which those inside [lo, hi) count.
__device__ __forceinline__ void load_keys(const float* __restrict__ srow, int first4, int lo, int hi, uint32_t (&key)[4],
                                          bool (&in)[4])
{
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (first4 < hi) v = *reinterpret_cast<const float4*>(srow + first4);     // row stride is a multiple of 64: in bounds
    const float f[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        in[i] = first4 + i >= lo && first4 + i < hi;
        key[i] = score_key(f[i]);
    }
}

// The later passes work on chunks that start at a multiple of 4 positions (lo4), which can add one chunk.
__device__ __forceinline__ int chunks_from_lo4(const RepDev& rd)
{
    return (rd.hi - (rd.lo & ~3) + HC_SEL_CHUNK - 1) / HC_SEL_CHUNK;
}

// PASS 2: digit two (bits 20..10) among keys whose first digit matches; PASS 3: digit three (bits 9..0)
// among keys whose upper 22 bits match.  One workgroup handles every set size of its pivot: wave ks
// finds the digit of set size ks, then all waves histogram their candidates for each set size.
template <int PASS>
__global__ __launch_bounds__(BLK, 8) void mon_hist(MonBatch B, int span)
{
    extern __shared__ uint32_t sh[];              // [nk][HC_RADIX_BINS]
    __shared__ uint32_t sm_prefix[HC_MAX_K_PER_REP];
    const MonItem& it = B.it[blockIdx.z];
    const int rep = blockIdx.y;
    if (rep >= it.n_reps || mon_skip(it, rep)) return;
    const Ws ws = it.ws;
    const RepDev* __restrict__ reps = it.reps;
    const float* __restrict__ scores = it.scores;
    const RepDev rd = reps[rep];
    const int lo4 = rd.lo & ~3;
    const int nchunk = chunks_from_lo4(rd);
    const int c0 = blockIdx.x * span, c1 = min(c0 + span, nchunk);
    if (c0 >= nchunk) return;
    const RepWs w = ws.rep(rep);
    for (int i = threadIdx.x; i < rd.nk * HC_RADIX_BINS; i += BLK) sh[i] = 0u;

    for (int ks = threadIdx.x >> 6; ks < rd.nk; ks += NWAVE) {     // one wave per set size
        uint32_t prefix, remaining;
        if (PASS == 2) {
            find_digit_wave<HC_RADIX_BINS>(w.h1, (uint32_t)reps[rep].k[ks], prefix, remaining);   // (indexing the register copy would spill it)
        } else {
            uint32_t d2;
            find_digit_wave<HC_RADIX_BINS>(w.h2 + (size_t)ks * HC_RADIX_BINS, w.sel[ks * 4 + 1], d2, remaining);
            prefix = (w.sel[ks * 4 + 0] << 11) | d2;
        }
        if ((threadIdx.x & 63) == 0) {
            sm_prefix[ks] = prefix;
            if (blockIdx.x == 0) {   // state for the next pass (every workgroup computes the same value)
                w.sel[ks * 4 + (PASS == 2 ? 0 : 2)] = prefix;
                w.sel[ks * 4 + (PASS == 2 ? 1 : 3)] = remaining;
            }
        }
    }
    __syncthreads();
    const float* srow = scores + (size_t)rep * ws.max_ctx;
    for (int ch = c0; ch < c1; ch += 2) {         // two chunks' loads in flight
        uint32_t key[2][4];
        bool in[2][4];
        load_keys(srow, lo4 + ch * HC_SEL_CHUNK + threadIdx.x * 4, rd.lo, rd.hi, key[0], in[0]);
        load_keys(srow, lo4 + (ch + 1) * HC_SEL_CHUNK + threadIdx.x * 4, rd.lo, ch + 1 < c1 ? rd.hi : 0, key[1], in[1]);
        for (int ks = 0; ks < rd.nk; ++ks) {
            const uint32_t prefix = sm_prefix[ks];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (!in[u][i]) continue;
                    if (PASS == 2) {
                        if ((key[u][i] >> 21) == prefix) atomicAdd(&sh[ks * HC_RADIX_BINS + ((key[u][i] >> 10) & 0x7ffu)], 1u);
                    } else {
                        if ((key[u][i] >> 10) == prefix) atomicAdd(&sh[ks * HC_RADIX_BINS + (key[u][i] & 0x3ffu)], 1u);
                    }
                }
            }
        }
    }
    __syncthreads();
    uint32_t* gh = PASS == 2 ? w.h2 : w.h3;
    for (int i = threadIdx.x; i < rd.nk * HC_RADIX_BINS; i += BLK)
        if (sh[i]) atomicAdd(&gh[i], sh[i]);
}

// Keys of the 16 consecutive candidates of a lane (positions first16 .. first16+15, first16 a multiple of 4:
// four 16-byte loads) and the mask of those inside [lo, hi).  One wave covers a chunk this way, in position
// order, so the ordered passes below need no workgroup barriers.
__device__ __forceinline__ void load_keys16(const float* __restrict__ srow, int first16, int lo, int hi, uint32_t (&key)[16],
                                            uint32_t& inmask)
{
    float4 v[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        v[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (first16 + 4 * q < hi) v[q] = *reinterpret_cast<const float4*>(srow + first16 + 4 * q);   // row stride is a multiple of 64: in bounds
    }
    inmask = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float f[4] = {v[q].x, v[q].y, v[q].z, v[q].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j = first16 + 4 * q + i;
            if (j >= lo && j < hi) inmask |= 1u << (4 * q + i);
            key[4 * q + i] = score_key(f[i]);
        }
    }
}

// Finds the threshold key of every set size, then per chunk the counts of greater and of equal keys.
// Wave v of the workgroup takes the chunks c0 + v, c0 + v + 4, ... of the workgroup's span.
__global__ __launch_bounds__(BLK) void mon_count(MonBatch B, int span, int G)
{
    __shared__ uint32_t sm_tau[HC_MAX_K_PER_REP];
    const MonItem& it = B.it[blockIdx.z];
    const int rep = blockIdx.y;
    if (rep >= it.n_reps || mon_skip(it, rep)) return;
    const Ws ws = it.ws;
    const RepDev* __restrict__ reps = it.reps;
    const float* __restrict__ scores = it.scores;
    const RepDev rd = reps[rep];
    const int lo4 = rd.lo & ~3;
    const int nchunk = chunks_from_lo4(rd);
    const int c0 = blockIdx.x * span, c1 = min(c0 + span, nchunk);
    if (c0 >= nchunk) return;
    const RepWs w = ws.rep(rep);
    const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int ks = wv; ks < rd.nk; ks += NWAVE) {
        uint32_t d3, need;
        find_digit_wave<1024>(w.h3 + (size_t)ks * HC_RADIX_BINS, w.sel[ks * 4 + 3], d3, need);
        const uint32_t tau = (w.sel[ks * 4 + 2] << 10) | d3;
        if (lane == 0) {
            sm_tau[ks] = tau;
            // The first workgroup leaves tau / need for mon_write in the first two words, which this
            // kernel does not read (words 2 and 3 are still being read by the other workgroups).
            if (blockIdx.x == 0) {
                w.sel[ks * 4 + 0] = tau;
                w.sel[ks * 4 + 1] = need;
            }
        }
    }
    __syncthreads();
    if (it.need_sense == 0 && blockIdx.x == 0 && threadIdx.x == 0) {
        // The check of this step's filter.  The split pass dropped the rows whose statistic sum_g 2^(t_g - ref_g)
        // stayed below cutsum; with this step's own log-sum-exp such a row's score is below
        // (cutsum / G) max_g 2^(ref_g - lse_g).  If even the smallest list threshold found among the kept rows
        // reaches that bound (with room for the rounding of the statistic), no dropped row belongs to any list and
        // the lists are those of all rows.  Otherwise the dense passes redo this pivot from all of its logits.
        const RepFilter f = it.filt[rep];
        if (f.cutsum > 0.f) {
            uint32_t tmin = sm_tau[0];
            for (int ks = 1; ks < rd.nk; ++ks) tmin = min(tmin, sm_tau[ks]);
            float delta = 0.f;
            for (int g = 0; g < G; ++g) delta = fmaxf(delta, exp2f(f.ref[g] - it.lse[(size_t)rd.bh * G + g] * 1.4426950408889634f));
            const float bound = f.cutsum / (float)G * delta * 1.0001f;
            if (!(key_score(tmin) >= bound)) it.need_w[rep] = 5;
        }
    }
    const float* srow = scores + (size_t)rep * ws.max_ctx;
    for (int ch = c0 + wv; ch < c1; ch += NWAVE) {
        uint32_t key[16], inmask;
        load_keys16(srow, lo4 + ch * HC_SEL_CHUNK + lane * 16, rd.lo, rd.hi, key, inmask);
        for (int ks = 0; ks < rd.nk; ++ks) {
            const uint32_t tau = sm_tau[ks];
            uint32_t gt = 0, eq = 0;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const bool in = (inmask >> i) & 1u;
                gt += in && key[i] > tau;
                eq += in && key[i] == tau;
            }
            for (int o = 32; o > 0; o >>= 1) {
                gt += __shfl_xor(gt, o);
                eq += __shfl_xor(eq, o);
            }
            if (lane == 0) {
                w.cnt[((size_t)ks * ws.max_chunks + ch) * 2 + 0] = gt;
                w.cnt[((size_t)ks * ws.max_chunks + ch) * 2 + 1] = eq;
            }
        }
    }
}

struct DriftCfg {
    int window, metric, tau_num, tau_den, max_k, tumbling;
};

// Keys of the 8 consecutive candidates of a lane (two 16-byte loads) and the mask of those inside [lo, hi).
__device__ __forceinline__ void load_keys8(const float* __restrict__ srow, int first8, int lo, int hi, uint32_t (&key)[8],
                                           uint32_t& inmask)
{
    float4 v[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        v[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (first8 + 4 * q < hi) v[q] = *reinterpret_cast<const float4*>(srow + first8 + 4 * q);   // row stride is a multiple of 64: in bounds
    }
    inmask = 0;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const float f[4] = {v[q].x, v[q].y, v[q].z, v[q].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j = first8 + 4 * q + i;
            if (j >= lo && j < hi) inmask |= 1u << (4 * q + i);
            key[4 * q + i] = score_key(f[i]);
        }
    }
}

// Ordered compaction of the index lists of one pivot (blockIdx.y) into topk_idx, and |T ∩ baseline| for the
// monitored list.  Wave v takes the chunks c0 + v, c0 + v + 4, ... of the workgroup's span, each as two halves of
// 512 candidates in position order (8 per lane), and reads a half's keys once for all set sizes; what a set size
// carries from half to half (equal keys seen, entries emitted) lives in LDS: the kernel has to fit, in registers,
// beside the attention pass's waves on a compute unit.  Lists of equal size (satellites with the same budget)
// share the selection and differ only in the row they are written to.  No workgroup barriers.
__global__ __launch_bounds__(BLK, 8) void mon_write(MonBatch B, DriftCfg cfg, int span)
{
    __shared__ uint32_t sm_carry[NWAVE][HC_MAX_K_PER_REP][2];      // per wave and set size: equal keys before, entries emitted
    const MonItem& it = B.it[blockIdx.z];
    const int rep = blockIdx.y;
    if (rep >= it.n_reps || mon_skip(it, rep)) return;
    const Ws ws = it.ws;
    const RepDev* __restrict__ reps = it.reps;
    const OutDev* __restrict__ outs = it.outs;
    const int32_t* __restrict__ pmap = it.pos_map ? it.pos_map + (size_t)rep * ws.max_ctx : nullptr;
    const float* __restrict__ scores = it.scores;
    int32_t* __restrict__ topk_idx = it.topk_idx;
    const RepDev rd = reps[rep];
    const int lo4 = rd.lo & ~3;
    const int nchunk = chunks_from_lo4(rd);
    const int c0 = blockIdx.x * span, c1 = min(c0 + span, nchunk);
    if (c0 >= nchunk) return;
    const RepWs w = ws.rep(rep);
    const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const float* srow = scores + (size_t)rep * ws.max_ctx;

    for (int chunk = c0 + wv; chunk < c1; chunk += NWAVE) {
        for (int ks = 0; ks < rd.nk; ++ks) {
            const uint32_t need = w.sel[ks * 4 + 1];
            const uint32_t* cnt = w.cnt + (size_t)ks * ws.max_chunks * 2;
            // Prefix over the chunks before this one: equal-keyed candidates seen, and list entries emitted.  A
            // chunk emits all its greater keys plus as many equal keys as are still needed.
            uint32_t eq_before = 0, emitted = 0;
            for (int b0 = 0; b0 < chunk; b0 += 64) {
                const int b = b0 + lane;
                const uint32_t g = b < chunk ? cnt[b * 2] : 0u, e = b < chunk ? cnt[b * 2 + 1] : 0u;
                uint32_t etot;
                const uint32_t eprev = eq_before + wave_exscan(e, etot);
                const uint32_t left = need > eprev ? need - eprev : 0u;
                uint32_t mine = g + (e < left ? e : left);
                for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o);
                emitted += mine;
                eq_before += etot;
            }
            if (lane == 0) {
                sm_carry[wv][ks][0] = eq_before;
                sm_carry[wv][ks][1] = emitted;
            }
        }
        uint32_t hits = 0;
        for (int half = 0; half < 2; ++half) {
            uint32_t key[8], inmask;
            const int first8 = lo4 + chunk * HC_SEL_CHUNK + half * (HC_SEL_CHUNK / 2) + lane * 8;
            load_keys8(srow, first8, rd.lo, rd.hi, key, inmask);
            // the positions of the lane's 8 rows: themselves, or (rows a filtering split pass kept) what the map says
            int32_t jj[8];
            if (pmap) {
                int4 pa = make_int4(0, 0, 0, 0), pb = pa;
                if (first8 < rd.hi) pa = *reinterpret_cast<const int4*>(pmap + first8);          // (row stride a multiple of 64: in bounds)
                if (first8 + 4 < rd.hi) pb = *reinterpret_cast<const int4*>(pmap + first8 + 4);
                jj[0] = pa.x; jj[1] = pa.y; jj[2] = pa.z; jj[3] = pa.w;
                jj[4] = pb.x; jj[5] = pb.y; jj[6] = pb.z; jj[7] = pb.w;
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) jj[i] = first8 + i;
            }
            for (int ks = 0; ks < rd.nk; ++ks) {
                const uint32_t tau = w.sel[ks * 4 + 0], need = w.sel[ks * 4 + 1];
                const int k = reps[rep].k[ks];               // (indexing the register copy would spill it)
                const uint32_t eq_before = sm_carry[wv][ks][0], emitted = sm_carry[wv][ks][1];      // (written by this wave)
                uint32_t my_eq = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) my_eq += ((inmask >> i) & 1u) && key[i] == tau;
                uint32_t eq_tot;
                uint32_t eq_rank = eq_before + wave_exscan(my_eq, eq_tot);
                uint32_t selmask = 0, my_sel = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    if (!((inmask >> i) & 1u)) continue;
                    bool sel = key[i] > tau;
                    if (key[i] == tau) {
                        sel = eq_rank < need;
                        ++eq_rank;
                    }
                    if (sel) {
                        selmask |= 1u << i;
                        ++my_sel;
                    }
                }
                uint32_t sel_tot;
                const uint32_t pos0 = emitted + wave_exscan(my_sel, sel_tot);
                if (lane == 0) {
                    sm_carry[wv][ks][0] = eq_before + eq_tot;
                    sm_carry[wv][ks][1] = emitted + sel_tot;
                }
                if (ks == 0) {
                    // |T ∩ baseline| of the monitored list (set size 0): the bitmap words of the selected rows, all
                    // loads issued together (a row that is not selected reads word 0 and does not count)
                    uint32_t wd[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) wd[i] = w.bitmap[((selmask >> i) & 1u) ? (jj[i] >> 5) : 0];
#pragma unroll
                    for (int i = 0; i < 8; ++i) hits += ((selmask >> i) & 1u) & (wd[i] >> (jj[i] & 31));
                }
                for (int o = rd.out_begin; o < rd.out_begin + rd.out_count; ++o) {      // the rows this list goes to
                    const OutDev od = outs[o];
                    if (od.kslot != ks) continue;
                    int32_t* dst = topk_idx + (size_t)od.row * cfg.max_k;
                    uint32_t pos = pos0;
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        if (selmask & (1u << i)) {
                            if (pos < (uint32_t)k) dst[pos] = jj[i];     // pos < k always holds; the guard keeps a corrupt state in bounds
                            ++pos;
                        }
                    }
                }
            }
        }
        // Per-chunk hit counts of the monitored list, summed by mon_decide: hundreds of atomics on one word would serialise.
        for (int o2 = 32; o2 > 0; o2 >>= 1) hits += __shfl_xor(hits, o2);
        if (lane == 0) ws.hits[(size_t)rep * (ws.max_chunks + 1) + chunk] = hits;
    }
}

// Leaves a pivot's histograms and baseline bitmap clear for the next call.
__device__ __forceinline__ void clear_rep_ws(const RepWs& w, int hi)
{
    uint4* h4 = reinterpret_cast<uint4*>(w.h1);
    for (int i = threadIdx.x; i < (1 + 2 * HC_MAX_K_PER_REP) * HC_RADIX_BINS / 4; i += BLK) h4[i] = make_uint4(0u, 0u, 0u, 0u);
    for (int i = threadIdx.x; i < (hi + 31) / 32; i += BLK) w.bitmap[i] = 0u;
}

// One workgroup per pivot, after mon_write has completed (the kernel boundary makes its lists and the
// intersection count visible): window update, decision, baseline update.
__global__ __launch_bounds__(BLK) void mon_decide(MonBatch B, DriftCfg cfg, int G)
{
    const MonItem& it = B.it[blockIdx.y];
    if ((int)blockIdx.x >= it.n_reps) return;
    const Ws ws = it.ws;
    const RepDev* __restrict__ reps = it.reps;
    const int32_t* __restrict__ topk_idx = it.topk_idx;
    int32_t* __restrict__ base_idx = it.base_idx;
    int32_t* __restrict__ ring = it.ring;
    int32_t* __restrict__ inter_out = it.inter;
    int32_t* __restrict__ flag_out = it.flag;
    // The lower median is found by ranking (no local arrays: they would live in scratch memory, and a
    // kernel that needs scratch is far slower to launch).
    __shared__ int32_t sm_ring[HC_MAX_WINDOW];
    __shared__ int32_t sm_med;
    __shared__ int32_t sm_trig;
    const RepDev rd = reps[blockIdx.x];
    const int real_hi = it.real_reps[blockIdx.x].hi;     // the bitmap is indexed by position
    if (it.need_sense >= 0) {
        const bool need = it.need_r[blockIdx.x] != 0;
        if (it.need_sense == 1 && !need) return;          // the filtered chain decided: nothing to redo
        if (it.need_sense == 0 && need) {                  // the dense chain decides; it starts from a clear workspace
            clear_rep_ws(ws.rep(blockIdx.x), real_hi);
            return;
        }
    }
    const int k = rd.k[0];
    int32_t* rg = ring + (size_t)rd.bh * (cfg.window + 1);
    int n = rg[0];
    if (n < 0 || n > cfg.window) n = 0;
    const int drop = n == cfg.window ? 1 : 0;        // sliding window: the oldest value leaves
    __shared__ uint32_t sm_hits[NWAVE];
    {
        const int lo4 = rd.lo & ~3;
        const int nchunk = (rd.hi - lo4 + HC_SEL_CHUNK - 1) / HC_SEL_CHUNK;
        uint32_t h = 0;
        for (int c = threadIdx.x; c < nchunk; c += BLK) h += ws.hits[(size_t)blockIdx.x * (ws.max_chunks + 1) + c];
        for (int o = 32; o > 0; o >>= 1) h += __shfl_xor(h, o);
        if ((threadIdx.x & 63) == 0) sm_hits[threadIdx.x >> 6] = h;
        __syncthreads();
    }
    const int32_t inter = (int32_t)(sm_hits[0] + sm_hits[1] + sm_hits[2] + sm_hits[3]);
    if (it.store_slot != -1) {
        // >= 0: a buffered query of the window scored again at the test step (Algorithm 1): its overlap replaces
        // the one stored when the query was current.  Only while the ring is one short of full, i.e. the
        // monitor call that follows is the one that tests.  -2: the lists were all that was wanted.
        if (threadIdx.x == 0 && it.store_slot >= 0 && n == cfg.window - 1 && it.store_slot < n) rg[1 + it.store_slot] = inter;
        clear_rep_ws(ws.rep(blockIdx.x), real_hi);
        return;
    }
    const int m = n - drop + 1;                      // values in the window after the push
    if ((int)threadIdx.x < m) sm_ring[threadIdx.x] = (int)threadIdx.x == m - 1 ? inter : rg[1 + drop + threadIdx.x];
    __syncthreads();
    if ((int)threadIdx.x < m) {
        const int32_t v = sm_ring[threadIdx.x];
        int rank = 0;
        for (int j = 0; j < m; ++j) rank += sm_ring[j] < v || (sm_ring[j] == v && j < (int)threadIdx.x);
        if (rank == (m - 1) / 2) sm_med = v;         // lower median
    }
    __syncthreads();
    if ((int)threadIdx.x < m) rg[1 + threadIdx.x] = sm_ring[threadIdx.x];
    if (threadIdx.x == 0) {
        int trig = 0;
        if (m == cfg.window) {
            const long long med = sm_med;
            const long long kk = k;
            if (cfg.metric == HC_METRIC_OVERLAP)
                trig = med * cfg.tau_den < (long long)cfg.tau_num * kk;                     // med/k < tau
            else
                trig = med * cfg.tau_den < (long long)cfg.tau_num * (2 * kk - med);         // med/(2k-med) < tau
        }
        // the window restarts after a retrieval; a tumbling window after every test
        rg[0] = (trig || (cfg.tumbling && m == cfg.window)) ? 0 : m;
        inter_out[rd.bh] = inter;
        flag_out[rd.bh] = trig;
        sm_trig = trig;
        if (it.counts) {
            uint32_t* cn = it.counts + (size_t)blockIdx.x * 4;
            cn[0] += m == cfg.window;
            cn[1] += (uint32_t)trig;
            cn[2] += it.need_sense == 1;
            cn[3] = it.need_sense == 0 ? (uint32_t)rd.hi : 0xffffffffu;
        }
        if (it.filt) {
            // The filter of the next step's split pass: rows whose statistic, taken against this step's
            // log-sum-exp, stays below the smallest list threshold of this step divided by the margin are dropped.
            const RepWs w = ws.rep(blockIdx.x);
            uint32_t tmin = w.sel[0];                  // (mon_count left every set size's threshold key in word 0)
            for (int ks = 1; ks < rd.nk; ++ks) tmin = min(tmin, w.sel[ks * 4]);
            const float tau = key_score(tmin);
            RepFilter f;
            f.cutsum = (tau > 0.f && tau < 1.0e30f && it.margin >= 1.f) ? (float)G * tau / it.margin : 0.f;
            for (int g = 0; g < 8; ++g) f.ref[g] = g < G ? it.lse[(size_t)rd.bh * G + g] * 1.4426950408889634f : 0.f;
            f.armed = 1;
            for (int i = 0; i < 6; ++i) f.pad[i] = 0;
            it.filt[blockIdx.x] = f;
        }
    }
    __syncthreads();
    if (sm_trig) {                                   // K_base <- K_t
        const int32_t* src = topk_idx + (size_t)rd.bh * cfg.max_k;
        int32_t* base = base_idx + (size_t)rd.bh * cfg.max_k;
        for (int i = threadIdx.x; i < k; i += BLK) base[i] = src[i];
    }
    // every other kernel of this call is done with the histograms and the bitmap: leave them clear
    clear_rep_ws(ws.rep(blockIdx.x), real_hi);
}

// First pass of the selection over a pivot whose logits the split pass filtered: the rows it kept lie segment by
// segment in the pivot's block of rep_logits (positions in surv_pos, counts in seg_cnt).  They are scored with this
// step's log-sum-exp and laid out as one dense run in position order (scores[rep][0, n), dense_pos[rep][0, n)),
// over which the later passes then work as over a short context; the first-digit histogram and the baseline
// bitmap are made on the way, as in mon_score_hist.  Every workgroup makes the prefix sums of the pivot's
// segment counts itself (a few hundred numbers).
constexpr int MAX_FILTER_SEGS = 2048;
template <int G>
__global__ __launch_bounds__(BLK) void mon_sparse_score(MonBatch B, int max_k, int span)
{
    __shared__ uint32_t sh[HC_RADIX_BINS];
    __shared__ int sm_pref[MAX_FILTER_SEGS + 1];
    __shared__ int sm_row0[MAX_FILTER_SEGS];
    __shared__ int sm_wsum[NWAVE];
    __shared__ int sm_unknown;
    const MonItem& it = B.it[blockIdx.z];
    const int rep = blockIdx.y;
    if (rep >= it.n_reps) return;
    const Ws ws = it.ws;
    const RepDev rd = it.real_reps[rep];
    const HeadDev hd = it.heads[rd.bh];
    const int nseg = min(hd.part_count, MAX_FILTER_SEGS);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (threadIdx.x == 0) sm_unknown = 0;
    __syncthreads();
    int carry = 0;
    for (int base = 0; base < nseg; base += BLK) {
        const int sidx = base + threadIdx.x;
        int c = 0;
        if (sidx < nseg) {
            const SegDev sg = it.segs[hd.part_begin + sidx];
            c = it.seg_cnt[hd.part_begin + sidx];
            if (c < 0 || c > sg.row_end - sg.row_begin) {      // not a count the split pass can have written
                sm_unknown = 1;
                c = 0;
            }
            sm_row0[sidx] = sg.row_begin;
        }
        int inc = c;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(inc, o);
            if (lane >= o) inc += t;
        }
        if (lane == 63) sm_wsum[wv] = inc;
        __syncthreads();
        int before = carry;
        for (int k = 0; k < wv; ++k) before += sm_wsum[k];
        if (sidx < nseg) sm_pref[sidx] = before + inc - c;
        carry += sm_wsum[0] + sm_wsum[1] + sm_wsum[2] + sm_wsum[3];
        __syncthreads();
    }
    if (threadIdx.x == 0) sm_pref[nseg] = carry;
    const int n = carry;                                    // rows kept, all of them candidates
    int kmax = 0;
    for (int ks = 0; ks < rd.nk; ++ks) kmax = max(kmax, it.real_reps[rep].k[ks]);       // (indexing the register copy would spill it)
    // why a pivot goes to the dense passes: 1 more rows kept than the launch was sized for, 2 fewer than the longest
    // list needs, 3 a segment's count is out of range, 4 too many segments, (5: the check failed, below)
    const int why = sm_unknown != 0 ? 3 : hd.part_count > MAX_FILTER_SEGS ? 4 : n > it.cap_rows ? 1 : n < kmax ? 2 : 0;
    const bool bad = why != 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        // the pivot as the later passes see it: a context of n rows, all of them candidates
        RepDev* v = it.vreps + rep;
        v->bh = rd.bh;
        v->lo = 0;
        v->hi = bad ? 0 : n;
        v->nk = rd.nk;
        for (int ks = 0; ks < rd.nk; ++ks) v->k[ks] = it.real_reps[rep].k[ks];
        v->nchunk = bad ? 0 : (n + HC_SEL_CHUNK - 1) / HC_SEL_CHUNK;
        v->out_begin = rd.out_begin;
        v->out_count = rd.out_count;
        it.need_w[rep] = why;
    }
    if (bad) return;
    const int nchunk = (n + HC_SEL_CHUNK - 1) / HC_SEL_CHUNK;
    const int c0 = blockIdx.x * span, c1 = min(c0 + span, nchunk);
    if (c0 >= nchunk) return;
    const RepWs w = ws.rep(rep);
    for (int i = threadIdx.x; i < HC_RADIX_BINS; i += BLK) sh[i] = 0u;
    // baseline list -> bitmap (each active workgroup takes a slice of the list)
    const int32_t* basel = it.base_idx + (size_t)rd.bh * max_k;
    const int nblk = (nchunk + span - 1) / span;
    for (int i = blockIdx.x * BLK + threadIdx.x; i < rd.k[0]; i += nblk * BLK) {
        const int j = basel[i];
        if (j >= rd.lo && j < rd.hi) atomicOr(&w.bitmap[j >> 5], 1u << (j & 31));
    }
    __syncthreads();
    float l[G];
#pragma unroll
    for (int g = 0; g < G; ++g) l[g] = it.lse[(size_t)rd.bh * G + g];
    const float* lrow = it.rep_logits + (size_t)rep * G * ws.max_ctx;
    const int32_t* prow = it.surv_pos + (size_t)rep * ws.max_ctx;
    float* srow = it.scores + (size_t)rep * ws.max_ctx;
    int32_t* drow = it.dense_pos + (size_t)rep * ws.max_ctx;
    for (int ch = c0; ch < c1; ++ch) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int d = ch * HC_SEL_CHUNK + i * BLK + threadIdx.x;
            if (d >= n) continue;
            int lo = 0, hi = nseg;                             // the segment whose run holds kept row d
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (sm_pref[mid] <= d) lo = mid;
                else hi = mid;
            }
            const int src = sm_row0[lo] + (d - sm_pref[lo]);
            const float sc = score_of<G>(lrow, src, l, HC_AGG_PROB);
            srow[d] = sc;
            drow[d] = prow[src];
            atomicAdd(&sh[score_key(sc) >> 21], 1u);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < HC_RADIX_BINS; i += BLK)
        if (sh[i]) atomicAdd(&w.h1[i], sh[i]);
}

}   // namespace

// The launches of one chain of selection passes over a batch of layers.  mode 0: the plain chain (every pivot, all
// candidate positions).  mode 1: the chain over the rows a filtering split pass kept.  mode 2: the dense chain that
// stands by behind mode 1, for the pivots whose check failed.  ws_first: which workspace copy the first layer uses.
static hc_status run_chain(hc_ctx* ctx, int n, const hc_monitor_call* const* calls, int ws_first, int scores_given, int mode,
                           hipStream_t st)
{
    const hc_config& c = ctx->cfg;
    MonBatch B{};
    int max_reps = 0, max_nchunk = 0, max_nk = 0;
    for (int i = 0; i < n; ++i) {
        const hc_monitor_call& x = *calls[i];
        hc_monitor_ws& m = ctx->ws[ws_first + i];
        MonItem& it = B.it[i];
        it.ws = Ws{m.hist, m.sel, m.misc, m.cnt, m.bitmap, m.hits, ctx->max_chunks, c.max_ctx};
        it.reps = x.reps ? x.reps : x.L->reps;
        it.real_reps = it.reps;
        it.outs = x.reps ? x.outs : x.L->outs;
        it.rep_logits = x.rep_logits;
        it.lse = x.lse;
        it.scores = x.scores;
        it.topk_idx = x.topk_idx;
        it.base_idx = x.base_idx;
        it.ring = x.ring;
        it.inter = x.inter;
        it.flag = x.flag;
        it.n_reps = x.reps ? x.n_reps : x.L->n_reps;
        it.n_outs = x.reps ? x.n_outs : x.L->n_outs;
        it.store_slot = x.store_slot;
        it.need_sense = -1;
        if (!x.reps && x.store_slot == -1) it.counts = x.L->mon_counts;
        int nchunk = x.reps ? x.max_nchunk : x.L->max_nchunk;
        if (mode != 0) {
            const hc_layer* L = x.L;
            it.need_sense = mode == 1 ? 0 : 1;
            it.need_r = it.need_w = L->need;
            it.filt = L->filt;
            it.counts = L->mon_counts;
            it.margin = ctx->filter_margin;
            if (mode == 1) {
                it.reps = L->vreps;
                it.pos_map = it.dense_pos = L->dense_pos;
                it.heads = L->heads;
                it.segs = L->segs;
                it.seg_cnt = L->seg_cnt;
                it.surv_pos = L->surv_pos;
                it.vreps = L->vreps;
                // Once the filter is set few rows are kept (about 1.6 times the longest list at the usual margin of
                // 1.25); a step that keeps more is handed to the dense chain, so the launches need not be sized for
                // it, and every workgroup a launch does not have is one that does not queue for a compute unit.
                const int armed_cap = std::min(c.max_ctx, (ctx->filter_margin <= 1.5f ? 2 : 4) * L->max_k_any + 4096);
                it.cap_rows = L->filter_armed ? armed_cap : c.max_ctx;
                nchunk = std::min(nchunk, (it.cap_rows + HC_SEL_CHUNK - 1) / HC_SEL_CHUNK);
            }
        }
        max_reps = std::max(max_reps, it.n_reps);
        max_nchunk = std::max(max_nchunk, nchunk);
        max_nk = std::max(max_nk, x.reps ? x.max_nk : x.L->max_nk);
        if (m.dirty && mode != 2) {     // a previous call that used this workspace copy did not run to its last kernel
            mon_prep<<<dim3(16, ctx->max_reps), dim3(256), 0, st>>>(it.ws, c.max_ctx);
            HC_HIP(ctx, hipGetLastError());
        }
        m.dirty = true;
    }
    if (max_reps == 0) return HC_OK;
    // chunks per workgroup: aim at about 512 workgroups per launch, at most 8 chunks each
    // (the stand-by chain is there at every step and normally has nothing to do: few, long workgroups)
    const int span = mode == 2 ? 32
                               : ctx->monitor_span > 0 ? ctx->monitor_span : std::max(1, std::min(8, (n * max_reps * (max_nchunk + 1)) / 512));
    const dim3 g1((max_nchunk + span - 1) / span, max_reps, n);
    if (mode == 1) {
        switch (ctx->G) {
        case 1: mon_sparse_score<1><<<g1, dim3(BLK), hc_side_lds(ctx, (const void*)mon_sparse_score<1>, 0), st>>>(B, c.max_k, span); break;
        case 2: mon_sparse_score<2><<<g1, dim3(BLK), hc_side_lds(ctx, (const void*)mon_sparse_score<2>, 0), st>>>(B, c.max_k, span); break;
        case 4: mon_sparse_score<4><<<g1, dim3(BLK), hc_side_lds(ctx, (const void*)mon_sparse_score<4>, 0), st>>>(B, c.max_k, span); break;
        default: mon_sparse_score<8><<<g1, dim3(BLK), hc_side_lds(ctx, (const void*)mon_sparse_score<8>, 0), st>>>(B, c.max_k, span); break;
        }
    } else {
        switch (ctx->G) {
        case 1: mon_score_hist<1><<<g1, dim3(BLK), hc_side_lds(ctx, (const void*)mon_score_hist<1>, 0), st>>>(B, scores_given, c.agg, c.max_k, span); break;
        case 2: mon_score_hist<2><<<g1, dim3(BLK), hc_side_lds(ctx, (const void*)mon_score_hist<2>, 0), st>>>(B, scores_given, c.agg, c.max_k, span); break;
        case 4: mon_score_hist<4><<<g1, dim3(BLK), hc_side_lds(ctx, (const void*)mon_score_hist<4>, 0), st>>>(B, scores_given, c.agg, c.max_k, span); break;
        default: mon_score_hist<8><<<g1, dim3(BLK), hc_side_lds(ctx, (const void*)mon_score_hist<8>, 0), st>>>(B, scores_given, c.agg, c.max_k, span); break;
        }
    }
    HC_HIP(ctx, hipGetLastError());
    // the later passes start at a multiple of 4 positions, which can add one chunk
    const dim3 gk((max_nchunk + 1 + span - 1) / span, max_reps, n);
    const size_t hist_lds = (size_t)max_nk * HC_RADIX_BINS * sizeof(uint32_t);
    mon_hist<2><<<gk, dim3(BLK), hc_side_lds(ctx, (const void*)mon_hist<2>, (unsigned)hist_lds), st>>>(B, span);
    HC_HIP(ctx, hipGetLastError());
    mon_hist<3><<<gk, dim3(BLK), hc_side_lds(ctx, (const void*)mon_hist<3>, (unsigned)hist_lds), st>>>(B, span);
    HC_HIP(ctx, hipGetLastError());
    mon_count<<<gk, dim3(BLK), hc_side_lds(ctx, (const void*)mon_count, 0), st>>>(B, span, ctx->G);
    HC_HIP(ctx, hipGetLastError());
    DriftCfg dc{c.window, c.metric, c.tau_num, c.tau_den, c.max_k, c.window_mode != HC_WINDOW_SLIDING};
    // the write pass has no per-workgroup set-up to amortise: one chunk per wave
    const int span_w = mode == 2 ? 4 * NWAVE : NWAVE;
    mon_write<<<dim3((max_nchunk + 1 + span_w - 1) / span_w, max_reps, n), dim3(BLK), hc_side_lds(ctx, (const void*)mon_write, 0), st>>>(B, dc, span_w);
    HC_HIP(ctx, hipGetLastError());
    mon_decide<<<dim3(max_reps, n), dim3(BLK), hc_side_lds(ctx, (const void*)mon_decide, 0), st>>>(B, dc, ctx->G);
    HC_HIP(ctx, hipGetLastError());
    return HC_OK;
}

hc_status hc_launch_monitor(hc_ctx* ctx, int n, const hc_monitor_call* calls, int scores_given, hipStream_t st)
{
    if (n < 1 || n > HC_MAX_GROUP) return hc_fail(ctx, HC_EINVAL, "monitor batch of %d layers", n);
    // Layers whose split pass filtered the pivot logits are handled over the kept rows, with the dense chain behind
    // them; all others (and every call that brings its own scores or logits: given scores, the window's re-scored
    // queries, the prefill-time selection) by the plain chain.
    const hc_monitor_call* plain[HC_MAX_GROUP];
    const hc_monitor_call* filt[HC_MAX_GROUP];
    int n_plain = 0, n_filt = 0;
    for (int i = 0; i < n; ++i) {
        const hc_monitor_call& x = calls[i];
        const bool f = !scores_given && x.store_slot == -1 && x.reps == nullptr && hc_layer_filtered(ctx, x.L);
        if (f && !(x.arena ? x.arena : x.L->last_arena))
            return hc_fail(ctx, HC_ESTATE, "monitor of a filtering layer before any attention call with pivot logits");
        (f ? filt[n_filt++] : plain[n_plain++]) = &x;
    }
    hc_status s = HC_OK;
    if (n_plain > 0) s = run_chain(ctx, n_plain, plain, 0, scores_given, 0, st);
    if (s == HC_OK && n_filt > 0) {
        s = run_chain(ctx, n_filt, filt, n_plain, 0, 1, st);
        // behind it, for the pivots whose check failed (decided on the device; normally none): all logits over
        // again, then the plain passes over them
        if (s == HC_OK) {
            const hc_layer* layers[HC_MAX_GROUP];
            const void* arenas[HC_MAX_GROUP];
            float* logits[HC_MAX_GROUP];
            for (int i = 0; i < n_filt; ++i) {
                layers[i] = filt[i]->L;
                arenas[i] = filt[i]->arena ? filt[i]->arena : filt[i]->L->last_arena;
                logits[i] = const_cast<float*>(filt[i]->rep_logits);
            }
            s = hc_launch_rep_logits(ctx, n_filt, layers, arenas, logits, st);
        }
        if (s == HC_OK) s = run_chain(ctx, n_filt, filt, n_plain, 0, 2, st);
        if (s == HC_OK)
            for (int i = 0; i < n_filt; ++i) const_cast<hc_layer*>(filt[i]->L)->filter_armed = true;
    }
    if (s != HC_OK) return s;
    // everything enqueued: the workspace copies will be clear again when this call completes.  (Not so under
    // stream capture, where nothing has run yet and the graph may never be launched: they stay marked.)
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) != hipSuccess) cap = hipStreamCaptureStatusActive;
    if (cap == hipStreamCaptureStatusNone)
        for (int i = 0; i < n; ++i) ctx->ws[i].dirty = false;
    return HC_OK;
}

hc_status hc_monitor_set_lds_limit()
{
    // a pivot with HC_MAX_K_PER_REP distinct set sizes needs 64 KB of dynamic LDS for its histograms, on top of
    // the kernels' static LDS: above the default limit of 64 KB per workgroup; and beside the attention pass every
    // kernel here reserves more than half of a compute unit's LDS (hc_side_lds)
    const void* fns[] = {(const void*)mon_hist<2>, (const void*)mon_hist<3>, (const void*)mon_count, (const void*)mon_write,
                         (const void*)mon_decide, (const void*)mon_sparse_score<1>, (const void*)mon_sparse_score<2>,
                         (const void*)mon_sparse_score<4>, (const void*)mon_sparse_score<8>, (const void*)mon_score_hist<1>,
                         (const void*)mon_score_hist<2>, (const void*)mon_score_hist<4>, (const void*)mon_score_hist<8>};
    for (const void* fn : fns)
        if (hc_allow_lds(fn) != hipSuccess) return HC_EHIP;
    return HC_OK;
}
