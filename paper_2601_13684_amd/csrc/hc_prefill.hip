// hc_prefill.hip -- the state of a layer when decoding starts (Sec. 4.3, first paragraphs; Algorithm 1,
// stage 3 before the loop): C_GPU holds the full K/V of the full heads and, for every compressed head,
// the K/V of the positions with the head's own top attention scores of the prefill stage; C_CPU holds the
// satellites' whole K/V; K_base of every pivot is its top attended indices of the prefill stage.  The scores
// are the last prompt token's, averaged over the query group and optionally smoothed by a 1-D average
// pooling over positions (App. C.1).
//
// Steps, all on the caller's stream:
//   logits + lse of the last token against every selecting head's full K   (the contraction of hc_rescore.hip)
//   prefill_score_kernel   group mean of the softmax weights, then the pooling window           (below)
//   selection              the monitor's radix select + ordered compaction, lists only          (hc_monitor.hip)
//   prefill_place_kernel   rows of the resident positions -> the heads' blocks in the arena; baseline sets,
//                          slot maps and rings                                                  (below)
//   prefill_offload_kernel satellites' rows -> the pinned host tier, K row then V row per position (below)
#include "hc_internal.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int PF_BLK = 256;
constexpr int PF_CHUNK = 1024;       // positions per workgroup of the score kernel

// score[j] = (1/P) sum_{|d| <= P/2} a[j+d],  a[i] = (1/G) sum_g exp(l[i][g] - lse[g]) (or the mean logit), a = 0
// outside [0, ctx).  A workgroup stages a[] of its chunk and the halo in LDS, so every a[i] is computed once
// per workgroup; the window sum runs over increasing d, in fp32.
template <int G>
__global__ __launch_bounds__(PF_BLK) void prefill_score_kernel(const RepDev* __restrict__ reps, const HeadDev* __restrict__ heads,
                                                               const float* __restrict__ logits, const float* __restrict__ lse,
                                                               float* __restrict__ scores, int max_ctx, int agg, int pool)
{
    __shared__ float sm_a[PF_CHUNK + HC_MAX_POOL + 1];
    const int rep = blockIdx.y;
    const RepDev rd = reps[rep];
    const int ctx = heads[rd.bh].ctx;
    const int first = blockIdx.x * PF_CHUNK;
    if (first >= ctx) return;
    const int h = pool / 2;
    const float* lrow = logits + (size_t)rep * G * max_ctx;
    float l[G];
#pragma unroll
    for (int g = 0; g < G; ++g) l[g] = agg == HC_AGG_PROB ? lse[(size_t)rd.bh * G + g] : 0.f;
    for (int i = threadIdx.x; i < PF_CHUNK + 2 * h; i += PF_BLK) {
        const int j = first - h + i;
        float a = 0.f;
        if (j >= 0 && j < ctx) {
            float v[G];
            if (G == 1) {
                v[0] = lrow[j];
            } else if (G == 2) {
                const float2 t = reinterpret_cast<const float2*>(lrow)[j];
                v[0] = t.x; v[1] = t.y;
            } else {
#pragma unroll
                for (int q = 0; q < G / 4; ++q) {
                    const float4 t = reinterpret_cast<const float4*>(lrow)[(size_t)j * (G / 4) + q];
                    v[4 * q] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
                }
            }
            if (agg == HC_AGG_PROB) {
#pragma unroll
                for (int g = 0; g < G; ++g) a += expf(v[g] - l[g]);
            } else if (G == 4) {
                a = (v[0] + v[1]) + (v[2] + v[3]);
            } else {
#pragma unroll
                for (int g = 0; g < G; ++g) a += v[g];
            }
            a *= 1.0f / (float)G;
        }
        sm_a[i] = a;
    }
    __syncthreads();
    float* srow = scores + (size_t)rep * max_ctx;
    const float inv = 1.0f / (float)pool;
    for (int i = threadIdx.x; i < PF_CHUNK; i += PF_BLK) {
        const int j = first + i;
        if (j >= ctx) break;
        float s = sm_a[i + h];
        if (pool > 1) {
            s = 0.f;
            for (int d = 0; d < pool; ++d) s += sm_a[i + d];
            s *= inv;
        }
        srow[j] = s;
    }
}

// Slot i of a compressed head holds: i < sink: position i; then the last `recent` positions in order; then
// the selected positions in ascending order.  A full head holds all of its positions.  A workgroup takes
// tiles of 32 slots (1024 16-byte pieces; a row, K then V, is 32 consecutive pieces), tile x, x + gridDim.x,
// ... of its head; a thread moves four pieces of a tile, all four loads issued before the first store, so
// that a long head's copy has 16 KB per workgroup in flight.  Source rows are read once and destination
// rows are not read again by this call: streaming loads and stores.
__global__ __launch_bounds__(PF_BLK) void prefill_place_kernel(const HeadDev* __restrict__ heads, const PreSrc* __restrict__ src,
                                                               const RepDev* __restrict__ reps, const int32_t* __restrict__ rep_slot_of,
                                                               const uint4* __restrict__ kv_prefill, uint4* __restrict__ arena,
                                                               const int32_t* __restrict__ topk_idx, int32_t* __restrict__ base_idx,
                                                               int32_t* __restrict__ slot_pos, int32_t* __restrict__ ring, int max_k,
                                                               int window)
{
    const int bh = blockIdx.y;
    const HeadDev hd = heads[bh];
    const PreSrc s = src[bh];
    const int32_t* list = topk_idx + (size_t)bh * max_k;
    const int fixed = hd.sink + hd.recent;
    const bool full = hd.role == HC_ROLE_FULL;
    const int tiles = (hd.len + 31) / 32;
    const int piece = threadIdx.x & 31, row_in = threadIdx.x >> 5;        // 8 rows per quarter of a tile
    const bool isv = piece >= 16;
    const size_t from0 = (size_t)(isv ? s.v_off : s.k_off) / 8 + (piece & 15);
    const size_t to0 = (size_t)(isv ? hd.v_off : hd.k_off) / 8 + (piece & 15);
    for (int tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        u32x4 v[4];
        int slot[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            slot[u] = tile * 32 + u * 8 + row_in;
            int pos = slot[u];
            if (!full && slot[u] < hd.len) {
                if (slot[u] >= fixed) pos = list[slot[u] - fixed];
                else if (slot[u] >= hd.sink) pos = hd.ctx - hd.recent + (slot[u] - hd.sink);
                pos = min(max(pos, 0), hd.ctx - 1);               // a corrupt list cannot lead outside the head's rows
            }
            if (slot[u] < hd.len) v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kv_prefill) + from0 + (size_t)pos * 16);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (slot[u] < hd.len) __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4*>(arena) + to0 + (size_t)slot[u] * 16);
    }
    if (blockIdx.x != 0) return;
    // tables: the ring starts empty; a satellite's slot map names what its retrieved slots hold; a pivot's
    // baseline set is its own list
    for (int i = threadIdx.x; i <= window; i += PF_BLK) ring[(size_t)bh * (window + 1) + i] = 0;
    if (hd.role == HC_ROLE_SATELLITE && slot_pos) {
        for (int i = threadIdx.x; i < hd.len - fixed; i += PF_BLK) slot_pos[(size_t)bh * max_k + i] = list[i];
    }
    if (full && rep_slot_of[bh] >= 0) {
        const int k = reps[rep_slot_of[bh]].k[0];
        for (int i = threadIdx.x; i < k; i += PF_BLK) base_idx[(size_t)bh * max_k + i] = list[i];
    }
}

// The host tier's block of a satellite is [ctx][2][D]: piece idx of the block is piece idx % 16 of the K row
// (idx / 16 even) or V row (odd) of position idx / 32, so the stores of a wave are 1 KB contiguous.
__global__ __launch_bounds__(PF_BLK) void prefill_offload_kernel(const HeadDev* __restrict__ heads, const SatDev* __restrict__ sats,
                                                                 const PreSrc* __restrict__ src, const uint4* __restrict__ kv_prefill,
                                                                 uint4* __restrict__ tier)
{
    const int bh = sats[blockIdx.y].bh;
    const HeadDev hd = heads[bh];
    const PreSrc s = src[bh];
    const long long pieces = (long long)hd.ctx * 32;
    uint4* dst = tier + (size_t)hd.tier_off / 8;
    for (long long idx = (long long)blockIdx.x * PF_BLK + threadIdx.x; idx < pieces; idx += (long long)gridDim.x * PF_BLK) {
        const int pos = (int)(idx >> 5), piece = (int)(idx & 31);
        const size_t from = (size_t)(piece >= 16 ? s.v_off : s.k_off) / 8 + (size_t)pos * 16 + (piece & 15);
        dst[idx] = kv_prefill[from];
    }
}

size_t pf_align(size_t x) { return (x + 255) & ~(size_t)255; }

}   // namespace

hc_prefill_layout hc_prefill_plan(const hc_ctx* ctx, const hc_layer* L)
{
    const hc_config& c = ctx->cfg;
    const size_t n = (size_t)std::max(1, L->n_sel);
    hc_prefill_layout o{};
    size_t off = 0;
    o.logits_off = off;
    off += pf_align(n * c.max_ctx * ctx->G * 4);
    o.scores_off = off;
    off += pf_align(n * c.max_ctx * 4);
    o.lse_off = off;
    off += pf_align((size_t)c.B * c.Hq * 4);
    o.part_off = off;
    off += pf_align(n * HC_RESCORE_MAX_BLOCKS * 32 * 2 * 4);
    o.scratch_off = off;
    off += pf_align(2 * (size_t)c.B * c.Hkv * 4);
    o.bytes = off;
    return o;
}

hc_status hc_launch_prefill_scores(hc_ctx* ctx, const hc_layer* L, const float* logits, const float* lse, float* scores, int pool,
                                   hipStream_t st)
{
    if (L->n_sel == 0) return HC_OK;
    const hc_config& c = ctx->cfg;
    const dim3 grid((L->sel_max_len + PF_CHUNK - 1) / PF_CHUNK, L->n_sel);
    switch (ctx->G) {
    case 1: prefill_score_kernel<1><<<grid, dim3(PF_BLK), 0, st>>>(L->sel_reps, L->heads, logits, lse, scores, c.max_ctx, c.agg, pool); break;
    case 2: prefill_score_kernel<2><<<grid, dim3(PF_BLK), 0, st>>>(L->sel_reps, L->heads, logits, lse, scores, c.max_ctx, c.agg, pool); break;
    case 4: prefill_score_kernel<4><<<grid, dim3(PF_BLK), 0, st>>>(L->sel_reps, L->heads, logits, lse, scores, c.max_ctx, c.agg, pool); break;
    default: prefill_score_kernel<8><<<grid, dim3(PF_BLK), 0, st>>>(L->sel_reps, L->heads, logits, lse, scores, c.max_ctx, c.agg, pool); break;
    }
    HC_HIP(ctx, hipGetLastError());
    return HC_OK;
}

hc_status hc_launch_prefill_place(hc_ctx* ctx, const hc_layer* L, const void* kv_prefill, void* arena, void* tier,
                                  const int32_t* topk_idx, int32_t* base_idx, int32_t* slot_pos, int32_t* ring, hipStream_t st)
{
    const hc_config& c = ctx->cfg;
    int max_len = 1, max_ctx = 1;
    for (const hc_head_desc& h : L->hd_host) {
        max_len = std::max(max_len, (int)h.len);
        max_ctx = std::max(max_ctx, (int)h.ctx);
    }
    // Workgroups per head: the longest head's tiles of 32 rows, four to a workgroup (at most 2048); the
    // workgroups of a shorter head beyond its tiles exit at once.  Heads differ in length by up to the ratio of
    // context to budget, so a share per head by count would leave the chip to the few long heads' workgroups.
    const int max_tiles = (max_len + 31) / 32;
    const int per_head = std::max(1, std::min((max_tiles + 3) / 4, 2048));
    prefill_place_kernel<<<dim3(per_head, L->n_heads), dim3(PF_BLK), 0, st>>>(L->heads, L->pre_src, L->reps, L->rep_slot_dev,
                                                                               (const uint4*)kv_prefill, (uint4*)arena, topk_idx, base_idx,
                                                                               slot_pos, ring, c.max_k, c.window);
    HC_HIP(ctx, hipGetLastError());
    if (tier && L->n_sats > 0) {
        const int per_sat = std::max(1, std::min((max_ctx * 32 + PF_BLK * 8 - 1) / (PF_BLK * 8), std::max(1, 8 * ctx->n_cu / L->n_sats)));
        prefill_offload_kernel<<<dim3(per_sat, L->n_sats), dim3(PF_BLK), 0, st>>>(L->heads, L->sats, L->pre_src, (const uint4*)kv_prefill,
                                                                                   (uint4*)tier);
        HC_HIP(ctx, hipGetLastError());
    }
    return HC_OK;
}
