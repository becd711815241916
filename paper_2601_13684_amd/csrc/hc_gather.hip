// hc_gather.hip -- AsyncUpdate of Algorithm 1 (Sec. 4.3): C_GPU^(s) <- C_CPU^(s)[I_s].
//
// The host tier is pinned host memory that the kernels read directly over the host link, 512
// contiguous bytes per retrieved position (its K row followed by its V row), so no host thread has
// to learn which pivots fired: the predicate (flag of the satellite's pivot) is read on the device
// and workgroups of untriggered satellites leave at once.  32 lanes move one position: lanes 0-15
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

constexpr int ROWS_PER_PASS = 64;    // positions a workgroup has in flight: 8 per sub-pass, 8 sub-passes
constexpr int BLOCKS_PER_SAT = 16;   // workgroups per satellite: 1024 positions (512 KB) in flight per satellite;
                                     // few enough that an untriggered call costs next to nothing
constexpr int PLAN_THREADS = 1024;

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

__global__ __launch_bounds__(256) void gather_kernel(GatherBatch B, int max_k)
{
    const GatherItem& it = B.it[blockIdx.z];
    if ((int)blockIdx.y >= it.n_sats) return;
    const HeadDev* __restrict__ heads = it.heads;
    const uint16_t* __restrict__ tier = it.tier;
    uint16_t* __restrict__ arena = it.arena;
    const SatDev sd = it.sats[blockIdx.y];
    if (it.flag[sd.rep_bh] == 0) return;
    const HeadDev hd = heads[sd.bh];
    const bool delta = it.slot_pos != nullptr;
    const int32_t* pos_list = (delta ? it.pair_pos : it.topk_idx) + (size_t)sd.bh * max_k;
    const int32_t* slot_list = delta ? it.pair_slot + (size_t)sd.bh * max_k : nullptr;
    const int count = delta ? min(it.npairs[sd.bh], sd.r) : sd.r;
    const int sub = threadIdx.x >> 5;          // which of the 8 positions of a sub-pass
    const int l32 = threadIdx.x & 31;
    const int is_v = l32 >> 4;                 // lanes 16..31 move the V row
    const int chunk = l32 & 15;                // 16-byte chunk of the 256-byte row
    const u32x4* src_base = reinterpret_cast<const u32x4*>(tier + hd.tier_off);
    u32x4* dst_base = reinterpret_cast<u32x4*>(arena + (is_v ? hd.v_off : hd.k_off));
    for (int row_first = blockIdx.x * ROWS_PER_PASS; row_first < count; row_first += gridDim.x * ROWS_PER_PASS) {
        u32x4 buf[ROWS_PER_PASS / 8];
        int slot[ROWS_PER_PASS / 8];
#pragma unroll
        for (int p = 0; p < ROWS_PER_PASS / 8; ++p) {      // issue every host read first: they are latency-bound
            const int i = row_first + p * 8 + sub;
            slot[p] = -1;
            if (i < count) {
                const int j = pos_list[i];
                const int s = slot_list ? slot_list[i] : i;
                if (j >= 0 && j < hd.ctx && s >= 0 && s < sd.r) {     // a corrupt entry must not leave the tier block or the head's slots
                    buf[p] = __builtin_nontemporal_load(src_base + (size_t)j * 32 + is_v * 16 + chunk);
                    slot[p] = sd.first_slot + s;
                }
            }
        }
#pragma unroll
        for (int p = 0; p < ROWS_PER_PASS / 8; ++p)
            if (slot[p] >= 0) dst_base[(size_t)slot[p] * 16 + chunk] = buf[p];
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
        gather_plan_kernel<<<dim3(1, max_sats, n), dim3(PLAN_THREADS), lds, st>>>(B, max_k);
        HC_HIP(ctx, hipGetLastError());
    }
    const dim3 grid(std::min(BLOCKS_PER_SAT, (max_r + ROWS_PER_PASS - 1) / ROWS_PER_PASS), max_sats, n);
    gather_kernel<<<grid, dim3(256), 0, st>>>(B, max_k);
    HC_HIP(ctx, hipGetLastError());
    return HC_OK;
}

hc_status hc_gather_set_lds_limit()
{
    // the plan kernel may need more dynamic LDS than the default 64 KB limit
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gather_plan_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024);
    return e == hipSuccess ? HC_OK : HC_EHIP;
}
