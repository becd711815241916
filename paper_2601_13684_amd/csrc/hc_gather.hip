// hc_gather.hip -- AsyncUpdate of Algorithm 1 (Sec. 4.3): C_GPU^(s) <- C_CPU^(s)[I_s].
//
// The host tier is pinned host memory that the kernels read directly over the host link, 512
// contiguous bytes per retrieved position (its K row followed by its V row), so no host thread has
// to learn which pivots fired: the predicate (flag of the satellite's pivot) is read on the device
// and an untriggered call finds no rows to move.  32 lanes move one position: lanes 0-15
// the K row, lanes 16-31 the V row, 16 bytes each.
//
// The host link is the bound (about 55 GB/s against a refill of 10 MB per pivot), so with a slot map
// (slot_pos: which position every retrieved slot holds) only the difference moves: positions of the new
// list that are not resident go into the slots of resident positions that left the list.  The resident
// set afterwards is exactly the list; the order of the slots is not ascending any more, which attention
// does not care about.  gather_plan_kernel finds the difference, gather_kernel moves the rows.
#include <algorithm>

#include "hc_internal.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int GATHER_PASSES = 4;     // host reads a lane has in flight; a workgroup of T threads has T / 32 * 4 positions in flight
constexpr int GATHER_WORKGROUPS = 96; // workgroups of a gather launch, whatever the batch (measured at the 224K shape, batches
                                      // of 8 layers: 48 and fewer make the refill itself the bottleneck of the step, 128 and
                                      // more slow the attention pass that runs beside it; an untriggered call costs ~2 us)
constexpr int PLAN_THREADS = 256;      // (a larger workgroup does not find room on a compute unit beside the attention pass)

// One layer of a batched call (blockIdx.z picks the layer).
struct GatherItem {
    const SatDev* sats;
    const HeadDev* heads;
    const uint16_t* tier;
    const int32_t* topk_idx;
    const int32_t* flag;
    uint16_t* arena;
    int32_t* slot_pos;      // [B*Hkv][max_k] or nullptr: no slot map, the whole list is fetched in list order
    int32_t* pair_slot;     // [B*Hkv][max_k] workspace: the slots to overwrite ...
    int32_t* pair_pos;      // [B*Hkv][max_k]            ... and the positions that go there
    int32_t* npairs;        // [B*Hkv]
    int n_sats, pad;
};
struct GatherBatch {
    GatherItem it[HC_MAX_GROUP];
};

// Index of v in the ascending list a[0, n), or -1.
__device__ __forceinline__ int find_sorted(const int32_t* a, int n, int32_t v)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] < v) lo = mid + 1;
        else hi = mid;
    }
    return (lo < n && a[lo] == v) ? lo : -1;
}

// Exclusive prefix sums of two per-thread counts over the workgroup (PLAN_THREADS threads); totals returned.
__device__ __forceinline__ void block_exscan2(uint32_t a, uint32_t b, uint32_t* sm, uint32_t& ex_a, uint32_t& ex_b,
                                              uint32_t& tot_a, uint32_t& tot_b)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t ia = a, ib = b;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t ta = __shfl_up(ia, o), tb = __shfl_up(ib, o);
        if (lane >= o) {
            ia += ta;
            ib += tb;
        }
    }
    if (lane == 63) {
        sm[w * 2] = ia;
        sm[w * 2 + 1] = ib;
    }
    __syncthreads();
    uint32_t base_a = 0, base_b = 0;
    tot_a = tot_b = 0;
    for (int i = 0; i < PLAN_THREADS / 64; ++i) {
        if (i < w) {
            base_a += sm[i * 2];
            base_b += sm[i * 2 + 1];
        }
        tot_a += sm[i * 2];
        tot_b += sm[i * 2 + 1];
    }
    ex_a = base_a + ia - a;
    ex_b = base_b + ib - b;
}

// One workgroup per satellite: which slots hold positions that left the list (free), which positions of
// the list are not resident (fresh); the k-th free slot takes the k-th fresh position.  Dynamic LDS: the
// list (4 r bytes), found[r], keep[r].
__global__ __launch_bounds__(PLAN_THREADS) void gather_plan_kernel(GatherBatch B, int max_k)
{
    extern __shared__ int32_t sm_list[];
    __shared__ uint32_t sm_scan[2 * PLAN_THREADS / 64];
    const GatherItem& it = B.it[blockIdx.z];
    if ((int)blockIdx.y >= it.n_sats) return;
    const SatDev sd = it.sats[blockIdx.y];
    if (it.flag[sd.rep_bh] == 0) return;
    const int r = sd.r, tid = threadIdx.x;
    uint8_t* found = reinterpret_cast<uint8_t*>(sm_list + max_k);     // found[i]: list entry i is resident
    uint8_t* keep = found + max_k;                                     // keep[s]: slot s holds a listed position
    const int32_t* list = it.topk_idx + (size_t)sd.bh * max_k;
    int32_t* sp = it.slot_pos + (size_t)sd.bh * max_k;
    int32_t* pslot = it.pair_slot + (size_t)sd.bh * max_k;
    int32_t* ppos = it.pair_pos + (size_t)sd.bh * max_k;
    for (int i = tid; i < r; i += PLAN_THREADS) {
        sm_list[i] = list[i];
        found[i] = 0;
    }
    __syncthreads();
    for (int s = tid; s < r; s += PLAN_THREADS) {
        const int idx = find_sorted(sm_list, r, sp[s]);
        keep[s] = idx >= 0;
        if (idx >= 0) found[idx] = 1;       // a position held twice (a corrupt map) is caught by the count check below
    }
    __syncthreads();
    // each thread owns a contiguous run of slots / list entries, so that both compactions keep their order
    const int per = (r + PLAN_THREADS - 1) / PLAN_THREADS;
    const int e0 = min(r, tid * per), e1 = min(r, e0 + per);
    uint32_t n_free = 0, n_fresh = 0;
    for (int e = e0; e < e1; ++e) {
        n_free += !keep[e];
        n_fresh += !found[e];
    }
    uint32_t off_free, off_fresh, tot_free, tot_fresh;
    block_exscan2(n_free, n_fresh, sm_scan, off_free, off_fresh, tot_free, tot_fresh);
    if (tot_free != tot_fresh) {
        // the slot map does not describe a set of r distinct positions: start over from the list
        for (int i = tid; i < r; i += PLAN_THREADS) {
            pslot[i] = i;
            ppos[i] = sm_list[i];
            sp[i] = sm_list[i];
        }
        if (tid == 0) it.npairs[sd.bh] = r;
        return;
    }
    for (int e = e0; e < e1; ++e) {
        if (!keep[e]) pslot[off_free++] = e;
        if (!found[e]) ppos[off_fresh++] = sm_list[e];
    }
    __syncthreads();                        // the pairs are complete (and visible to the whole workgroup)
    for (int k = tid; k < (int)tot_free; k += PLAN_THREADS) sp[pslot[k]] = ppos[k];
    if (tid == 0) it.npairs[sd.bh] = (int32_t)tot_free;
}

// The rows to move, over all satellites of all layers of the batch, are numbered consecutively (satellite
// after satellite) and dealt to the workgroups in equal contiguous runs, so that the time does not depend on
// how unequal the satellites' lists are and a launch has as many workgroups as the host link needs, no more.
// Every workgroup makes the prefix sums of the satellites' row counts itself (a few hundred numbers).
// 32 lanes move one position (lanes 0-15 its K row, 16-31 its V row, 16 bytes each); a workgroup has
// ROWS_PER_PASS positions in flight.
constexpr int MAX_GATHER_SATS = 1024;     // satellites of a batch (layers x satellites per layer)
__global__ __launch_bounds__(256, 8) void gather_kernel(GatherBatch B, int n_items, int max_sats, int max_k)
{
    __shared__ int sm_start[MAX_GATHER_SATS + 1];
    __shared__ int sm_wsum[4];
    const int n_ent = n_items * max_sats;
    const int nthr = blockDim.x;            // 64, 128 or 256
    if (threadIdx.x < 4) sm_wsum[threadIdx.x] = 0;
    __syncthreads();
    // counts -> exclusive prefix sums (entry e = item e / max_sats, satellite e % max_sats)
    int carry = 0;
    for (int base = 0; base < n_ent; base += nthr) {
        const int e = base + threadIdx.x;
        int c = 0;
        if (e < n_ent) {
            const GatherItem& it = B.it[e / max_sats];
            const int sidx = e % max_sats;
            if (sidx < it.n_sats) {
                const SatDev sd = it.sats[sidx];
                if (it.flag[sd.rep_bh] != 0) c = it.slot_pos ? min(max(it.npairs[sd.bh], 0), sd.r) : sd.r;
            }
        }
        int inc = c;
        const int lane = threadIdx.x & 63;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(inc, o);
            if (lane >= o) inc += t;
        }
        if (lane == 63) sm_wsum[threadIdx.x >> 6] = inc;
        __syncthreads();
        int before = carry;
        for (int k = 0; k < (int)(threadIdx.x >> 6); ++k) before += sm_wsum[k];
        if (e < n_ent) sm_start[e] = before + inc - c;
        carry += sm_wsum[0] + sm_wsum[1] + sm_wsum[2] + sm_wsum[3];
        __syncthreads();
    }
    if (threadIdx.x == 0) sm_start[n_ent] = carry;
    __syncthreads();
    const int total = carry;
    if (total == 0) return;
    const int per = ((total + (int)gridDim.x - 1) / (int)gridDim.x + 7) & ~7;
    const int g_begin = blockIdx.x * per, g_end = min(total, g_begin + per);
    const int nsub = nthr >> 5;                // positions of a sub-pass
    const int sub = threadIdx.x >> 5;          // which of them this half-wave moves
    const int l32 = threadIdx.x & 31;
    const int is_v = l32 >> 4;                 // lanes 16..31 move the V row
    const int chunk = l32 & 15;                // 16-byte chunk of the 256-byte row
    for (int row_first = g_begin; row_first < g_end; row_first += nsub * GATHER_PASSES) {
        u32x4 buf[GATHER_PASSES];
        u32x4* dst[GATHER_PASSES];
#pragma unroll
        for (int p = 0; p < GATHER_PASSES; ++p) {          // issue every host read first: they are latency-bound
            const int g = row_first + p * nsub + sub;
            dst[p] = nullptr;
            if (g < g_end) {
                int lo = 0, hi = n_ent;                    // the entry whose run holds row g
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (sm_start[mid] <= g) lo = mid;
                    else hi = mid;
                }
                const GatherItem& it = B.it[lo / max_sats];
                const SatDev sd = it.sats[lo % max_sats];
                const HeadDev hd = it.heads[sd.bh];
                const int i = g - sm_start[lo];
                const bool delta = it.slot_pos != nullptr;
                const int j = (delta ? it.pair_pos : it.topk_idx)[(size_t)sd.bh * max_k + i];
                const int sl = delta ? it.pair_slot[(size_t)sd.bh * max_k + i] : i;
                if (j >= 0 && j < hd.ctx && sl >= 0 && sl < sd.r) {     // a corrupt entry must not leave the tier block or the head's slots
                    const u32x4* src = reinterpret_cast<const u32x4*>(it.tier + hd.tier_off);
                    buf[p] = __builtin_nontemporal_load(src + (size_t)j * 32 + is_v * 16 + chunk);
                    dst[p] = reinterpret_cast<u32x4*>(it.arena + (is_v ? hd.v_off : hd.k_off)) + (size_t)(sd.first_slot + sl) * 16 + chunk;
                }
            }
        }
#pragma unroll
        for (int p = 0; p < GATHER_PASSES; ++p)
            if (dst[p]) *dst[p] = buf[p];
    }
}

}   // namespace

hc_status hc_launch_gather(hc_ctx* ctx, int n, const hc_gather_call* calls, hipStream_t st)
{
    if (n < 1 || n > HC_MAX_GROUP) return hc_fail(ctx, HC_EINVAL, "gather batch of %d layers", n);
    GatherBatch B{};
    int max_r = 0, max_sats = 0;
    bool any_delta = false;
    const int max_k = ctx->cfg.max_k;
    const size_t rows = (size_t)ctx->cfg.B * ctx->cfg.Hkv;
    for (int i = 0; i < n; ++i) {
        const hc_gather_call& x = calls[i];
        GatherItem& it = B.it[i];
        it = GatherItem{x.L->sats, x.L->heads, (const uint16_t*)x.tier, x.topk_idx, x.flag, (uint16_t*)x.arena, x.slot_pos,
                        ctx->pair_slot + i * rows * max_k, ctx->pair_pos + i * rows * max_k, ctx->npairs + i * rows,
                        x.L->n_sats, 0};
        any_delta |= x.slot_pos != nullptr;
        max_r = std::max(max_r, x.L->max_r);
        max_sats = std::max(max_sats, x.L->n_sats);
    }
    if (max_sats == 0 || max_r == 0) return HC_OK;
    if (any_delta) {
        for (int i = 0; i < n; ++i)
            if (!calls[i].slot_pos) return hc_fail(ctx, HC_EINVAL, "hc_gather: in one batch either every layer has a slot map or none");
        const size_t lds = (size_t)max_k * (sizeof(int32_t) + 2);
        if (lds > 144 * 1024) return hc_fail(ctx, HC_ESHAPE, "hc_gather: max_k %d is too large for the slot-map path", max_k);
        gather_plan_kernel<<<dim3(1, max_sats, n), dim3(PLAN_THREADS), hc_side_lds(ctx, (const void*)gather_plan_kernel, (unsigned)lds), st>>>(B, max_k);
        HC_HIP(ctx, hipGetLastError());
    }
    // A few dozen workgroups keep the host link busy.  More do not make the refill faster, and every compute unit
    // that hosts gather waves has its memory pipeline filled with reads that take microseconds, behind which the
    // attention waves on the same unit queue (measured at the 224K shape with 16 workgroups per satellite in a
    // batch of 8 layers: the attention launch that ran beside a refill took 400 us instead of 45).
    if (n * max_sats > MAX_GATHER_SATS) return hc_fail(ctx, HC_ESHAPE, "hc_gather: more than %d satellites in a batch", MAX_GATHER_SATS);
    long long rows_max = 0;
    for (int i = 0; i < n; ++i) rows_max += (long long)calls[i].L->n_sats * calls[i].L->max_r;
    const int thr = ctx->gather_threads, in_flight = thr / 32 * GATHER_PASSES;
    const int nwg = (int)std::max<long long>(1, std::min<long long>(ctx->gather_workgroups, (rows_max + in_flight - 1) / in_flight));
    gather_kernel<<<dim3(nwg), dim3(thr), hc_side_lds(ctx, (const void*)gather_kernel, 0), st>>>(B, n, max_sats, max_k);
    HC_HIP(ctx, hipGetLastError());
    return HC_OK;
}

// the plan kernel may need more dynamic LDS than the default 64 KB limit, and beside the attention pass both kernels
// reserve more than half of a compute unit's LDS (hc_side_lds)
hc_status hc_gather_set_lds_limit()
{
    if (hc_allow_lds((const void*)gather_plan_kernel) != hipSuccess || hc_allow_lds((const void*)gather_kernel) != hipSuccess) return HC_EHIP;
    return HC_OK;
}
