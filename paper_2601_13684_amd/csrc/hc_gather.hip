// hc_gather.hip -- AsyncUpdate of Algorithm 1 (Sec. 4.3): C_GPU^(s) <- C_CPU^(s)[I_s].
//
// The host tier is pinned host memory that the kernel reads directly over the host link, 512
// contiguous bytes per retrieved position (its K row followed by its V row), so no host thread has
// to learn which pivots fired: the predicate (flag of the satellite's pivot) is read on the device
// and workgroups of untriggered satellites leave at once.  32 lanes move one position: lanes 0-15
// the K row, lanes 16-31 the V row, 16 bytes each.
#include <algorithm>

#include "hc_internal.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int ROWS_PER_PASS = 64;    // positions a workgroup has in flight: 8 per sub-pass, 8 sub-passes
constexpr int BLOCKS_PER_SAT = 16;   // workgroups per satellite: 1024 positions (512 KB) in flight per satellite;
                                     // few enough that an untriggered call costs next to nothing

// One layer of a batched call (blockIdx.z picks the layer).
struct GatherItem {
    const SatDev* sats;
    const HeadDev* heads;
    const uint16_t* tier;
    const int32_t* topk_idx;
    const int32_t* flag;
    uint16_t* arena;
    int n_sats, pad;
};
struct GatherBatch {
    GatherItem it[HC_MAX_GROUP];
};

__global__ __launch_bounds__(256) void gather_kernel(GatherBatch B, int max_k)
{
    const GatherItem& it = B.it[blockIdx.z];
    if ((int)blockIdx.y >= it.n_sats) return;
    const HeadDev* __restrict__ heads = it.heads;
    const uint16_t* __restrict__ tier = it.tier;
    const int32_t* __restrict__ topk_idx = it.topk_idx;
    uint16_t* __restrict__ arena = it.arena;
    const SatDev sd = it.sats[blockIdx.y];
    if (it.flag[sd.rep_bh] == 0) return;
    const HeadDev hd = heads[sd.bh];
    const int32_t* list = topk_idx + (size_t)sd.bh * max_k;
    const int sub = threadIdx.x >> 5;          // which of the 8 positions of a sub-pass
    const int l32 = threadIdx.x & 31;
    const int is_v = l32 >> 4;                 // lanes 16..31 move the V row
    const int chunk = l32 & 15;                // 16-byte chunk of the 256-byte row
    const u32x4* src_base = reinterpret_cast<const u32x4*>(tier + hd.tier_off);
    u32x4* dst_base = reinterpret_cast<u32x4*>(arena + (is_v ? hd.v_off : hd.k_off));
    for (int row_first = blockIdx.x * ROWS_PER_PASS; row_first < sd.r; row_first += gridDim.x * ROWS_PER_PASS) {
        u32x4 buf[ROWS_PER_PASS / 8];
        int slot[ROWS_PER_PASS / 8];
#pragma unroll
        for (int p = 0; p < ROWS_PER_PASS / 8; ++p) {      // issue every host read first: they are latency-bound
            const int i = row_first + p * 8 + sub;
            slot[p] = -1;
            if (i < sd.r) {
                const int j = list[i];
                if (j >= 0 && j < hd.ctx) {                // a corrupt list entry must not leave the tier block
                    buf[p] = __builtin_nontemporal_load(src_base + (size_t)j * 32 + is_v * 16 + chunk);
                    slot[p] = sd.first_slot + i;
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
    for (int i = 0; i < n; ++i) {
        const hc_gather_call& x = calls[i];
        B.it[i] = GatherItem{x.L->sats, x.L->heads, (const uint16_t*)x.tier, x.topk_idx, x.flag, (uint16_t*)x.arena,
                             x.L->n_sats, 0};
        max_r = std::max(max_r, x.L->max_r);
        max_sats = std::max(max_sats, x.L->n_sats);
    }
    if (max_sats == 0 || max_r == 0) return HC_OK;
    const dim3 grid(std::min(BLOCKS_PER_SAT, (max_r + ROWS_PER_PASS - 1) / ROWS_PER_PASS), max_sats, n);
    gather_kernel<<<grid, dim3(256), 0, st>>>(B, ctx->cfg.max_k);
    HC_HIP(ctx, hipGetLastError());
    return HC_OK;
}
