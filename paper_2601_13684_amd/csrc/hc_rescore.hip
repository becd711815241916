// hc_rescore.hip -- Algorithm 1's test at t mod W = 0, first half: the pivots' buffered queries of the
// window are scored again against the pivots' caches as they are now (Attention(q_k, C_GPU) in the loop
// over k = t-W+1 .. t).  The second half (top-k of each, overlap with the baseline) is the monitor's
// selection passes, run over these logits.
//
// For one pivot this is a skinny dense contraction, logits[(W-1) G, N] = Q [(W-1) G, 128] x K^T [128, N],
// followed by a row-wise log-sum-exp over all N positions: the one place on the decode path where the
// matrix cores fit.  It is still bound by memory (K is read once: 256 B per position; the logits written
// are 4 G bytes per position and query), so the kernel is shaped like the streaming attention pass and
// MFMA only replaces the dot-product arithmetic:
//   * up to 32 query rows (32 / G buffered queries) form the A operand of v_mfma_f32_32x32x16_bf16 and stay
//     in registers for the whole pass; a wave takes 32 positions at a time as the B operand;
//   * a wave reads its 32 K rows (8 KB) with fully coalesced 16-byte loads (each instruction covers four
//     whole rows), two tiles in flight in registers, and turns them into operand layout (lane = position,
//     8 consecutive dimensions per lane and instruction) through a private, padded LDS tile: no block
//     barriers in the loop;
//   * the accumulator layout puts G = 4 consecutive rows, i.e. the G heads of one query, into four
//     consecutive registers of a lane, so a lane stores the [position][G] logits of a query with one
//     16-byte store and half a wave writes 512 contiguous bytes, in the layout the monitor reads;
//   * running maximum and sum per row are kept per lane in registers (base-2 exponents) and merged once at
//     the end, into one partial per workgroup; a second small kernel merges the partials into the lse.
#include "hc_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int RS_BLK = 256;
constexpr int RS_NWAVE = RS_BLK / 64;
constexpr int RS_TILE = 32;                     // positions per wave and iteration
constexpr int RS_WG_TILE = RS_TILE * RS_NWAVE;  // positions per workgroup and iteration
constexpr int RS_ROWS = 32;                     // query rows of one pass (the MFMA's M)
constexpr int RS_LDS_ROW = 256 + 16;            // bytes per staged K row: padded, so that the operand reads of 16 lanes hit 64 different banks
constexpr float RS_LOG2E = 1.4426950408889634f;
constexpr float RS_LN2 = 0.6931471805599453f;
constexpr float RS_INV_SQRT_D = 0.08838834764831845f;   // 1/sqrt(128), the factor the attention pass applies
constexpr float RS_SLACK = 16.0f;               // a term of the running sum is at most 2^16 times the reference's
constexpr float RS_M_INIT = -1.0e30f;           // finite: (old - new) never is inf - inf

// One layer of a batched launch (blockIdx.z picks the layer): the layers of a hc_decode_step group reach the
// end of their windows together, and one launch over all their pivots amortises what a launch costs.
struct RescoreArgs {
    const HeadDev* heads;
    const RepDev* reps;
    const uint16_t* arena;
    const uint16_t* q_first;        // first buffered query of this pass, [n_items][B][Hq][D]
    size_t q_item_stride;           // elements
    float* logits;                  // [n_items][n_reps][max_ctx][G]
    size_t logits_item_stride;      // floats
    float* lse;                     // [n_items][B*Hq]
    size_t lse_item_stride;
    float* part;                    // [n_reps][nblk][RS_ROWS][2]: running maximum (base-2 exponent), sum
    const PreSrc* src;              // prefill-time use: the K rows of head bh are at arena + src[bh].k_off, all ctx of them
    int n_items, n_reps, max_ctx, nblk;
};
struct RescoreBatch {
    RescoreArgs it[HC_MAX_GROUP];
};

__device__ __forceinline__ void merge_ml(float& m, float& z, float mo, float zo)
{
    const float mn = fmaxf(m, mo);
    z = z * __builtin_amdgcn_exp2f(m - mn) + zo * __builtin_amdgcn_exp2f(mo - mn);
    m = mn;
}

template <int G>
__global__ __launch_bounds__(RS_BLK) void rescore_logits_kernel(RescoreBatch batch)
{
    const RescoreArgs& a = batch.it[blockIdx.z];
    if ((int)blockIdx.y >= a.n_reps) return;
    __shared__ __attribute__((aligned(16))) unsigned char sm_k[RS_NWAVE][RS_TILE * RS_LDS_ROW];
    __shared__ float sm_m[RS_NWAVE][RS_ROWS], sm_z[RS_NWAVE][RS_ROWS];

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int col = lane & 31, hh = lane >> 5;
    const int rep = blockIdx.y;
    const RepDev rd = a.reps[rep];
    const HeadDev hd = a.heads[rd.bh];
    // a pivot is a full head: all of its context, in the arena; at prefill time any head's full K, in the caller's buffer
    const int ctx = a.src ? hd.ctx : hd.len;
    const int64_t k_off = a.src ? a.src[rd.bh].k_off : hd.k_off;
    const int tiles = (ctx + RS_WG_TILE - 1) / RS_WG_TILE;
    const int per = (tiles + a.nblk - 1) / a.nblk;
    const int t0 = blockIdx.x * per, t1 = min(tiles, t0 + per);

    // A operand: query row `col` of the pass = head col % G of buffered query col / G; rows past the
    // last query are zero.  Slab s of the contraction covers dimensions 16 s .. 16 s + 15, of which this
    // lane holds 8 hh .. 8 hh + 7.
    bf16x8 qa[8];
    {
        const int item = col / G, g = col % G;
        const bool have = item < a.n_items;
        const uint4* qp = reinterpret_cast<const uint4*>(a.q_first + (size_t)(have ? item : 0) * a.q_item_stride +
                                                         ((size_t)rd.bh * G + g) * HC_D);
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            uint4 v = qp[2 * s + hh];
            if (!have) v = make_uint4(0u, 0u, 0u, 0u);
            qa[s] = __builtin_bit_cast(bf16x8, v);
        }
    }

    float m[16], z[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        m[v] = RS_M_INIT;
        z[v] = 0.f;
    }

    const unsigned char* Kb = reinterpret_cast<const unsigned char*>(a.arena + k_off);
    unsigned char* mine = sm_k[w];
    // coalesced load of a tile: instruction s, lane l -> row 4 s + l / 16, 16-byte piece l % 16
    const int lrow = lane >> 4, lpiece = lane & 15;
    auto load_tile = [&](u32x4 (&r)[8], int t) {
        const int p0 = t * RS_WG_TILE + w * RS_TILE;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int row = min(p0 + 4 * s + lrow, ctx - 1);          // rows past the end are clamped here and masked below
            r[s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(Kb + (size_t)row * 256 + lpiece * 16));
        }
    };

    // Two tiles are in flight per wave (register buffers A and B): tile t is staged and consumed while t + 1 is
    // on its way and t + 2 is requested.
    auto consume = [&](u32x4 (&buf)[8], int t) {
#pragma unroll
        for (int s = 0; s < 8; ++s)
            *reinterpret_cast<u32x4*>(mine + (4 * s + lrow) * RS_LDS_ROW + lpiece * 16) = buf[s];
        if (t + 2 < t1) load_tile(buf, t + 2);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();

        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const u32x4 kv = *reinterpret_cast<const u32x4*>(mine + col * RS_LDS_ROW + (2 * s + hh) * 16);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[s], __builtin_bit_cast(bf16x8, kv), acc, 0, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();                              // the tile is consumed: the next iteration may overwrite it

        // acc[v] = <query row 8 (v / 4) + 4 hh + v % 4, K row pos>
        const int pos = t * RS_WG_TILE + w * RS_TILE + col;
        const bool valid = pos < ctx;
        float lg[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) lg[v] = acc[v] * RS_INV_SQRT_D;
        // Running sums relative to a reference that only moves when some logit exceeds it by more than
        // RS_SLACK (in base-2 exponent units): decided for the whole wave, so the common case is one
        // exponential per logit and no rescaling.
        float x[16];
        bool over = false;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            x[v] = lg[v] * RS_LOG2E;
            over |= x[v] > m[v] + RS_SLACK;
        }
        if (__builtin_amdgcn_ballot_w64(valid && over)) {
            if (valid) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float mn = fmaxf(m[v], x[v]);
                    z[v] *= __builtin_amdgcn_exp2f(m[v] - mn);
                    m[v] = mn;
                }
            }
        }
        if (valid) {
#pragma unroll
            for (int v = 0; v < 16; ++v) z[v] += __builtin_amdgcn_exp2f(x[v] - m[v]);
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int row0 = 8 * v4 + 4 * hh;                     // first of this lane's 4 consecutive query rows
                if (G >= 4) {
                    const int item = row0 / G, g0 = row0 % G;
                    if (item < a.n_items) {
                        float* dst = a.logits + (size_t)item * a.logits_item_stride + ((size_t)rep * a.max_ctx + pos) * G + g0;
                        *reinterpret_cast<float4*>(dst) = make_float4(lg[4 * v4], lg[4 * v4 + 1], lg[4 * v4 + 2], lg[4 * v4 + 3]);
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int item = (row0 + e) / G, g = (row0 + e) % G;
                        if (item < a.n_items)
                            a.logits[(size_t)item * a.logits_item_stride + ((size_t)rep * a.max_ctx + pos) * G + g] = lg[4 * v4 + e];
                    }
                }
            }
        }
    };
    u32x4 bufA[8], bufB[8];
    if (t0 < t1) load_tile(bufA, t0);
    if (t0 + 1 < t1) load_tile(bufB, t0 + 1);
#pragma unroll 1
    for (int t = t0; t < t1; t += 2) {
        consume(bufA, t);
        if (t + 1 < t1) consume(bufB, t + 1);
    }

    // merge over the 32 positions a half-wave holds (the common reference first, then one rescaling per lane
    // and plain sums), then over the waves
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        float mm = m[v];
#pragma unroll
        for (int o = 1; o < 32; o <<= 1) mm = fmaxf(mm, __shfl_xor(mm, o));
        float zz = z[v] * __builtin_amdgcn_exp2f(m[v] - mm);
#pragma unroll
        for (int o = 1; o < 32; o <<= 1) zz += __shfl_xor(zz, o);
        m[v] = mm;
        z[v] = zz;
    }
    if (col == 0) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = 8 * (v / 4) + 4 * hh + (v % 4);
            sm_m[w][row] = m[v];
            sm_z[w][row] = z[v];
        }
    }
    __syncthreads();
    if (tid < RS_ROWS) {
        float mm = sm_m[0][tid], zz = sm_z[0][tid];
#pragma unroll
        for (int k = 1; k < RS_NWAVE; ++k) merge_ml(mm, zz, sm_m[k][tid], sm_z[k][tid]);
        float* p = a.part + (((size_t)rep * a.nblk + blockIdx.x) * RS_ROWS + tid) * 2;
        p[0] = mm;
        p[1] = zz;
    }
}

// lse of every (buffered query, head of the pivot's group) from the workgroups' partials.  All loads of
// a thread are independent (the maximum first, then the sum relative to it), so the kernel costs a few
// memory round trips, not one per partial.
constexpr int RS_LSE_BLK = 1024;
constexpr int RS_LSE_SLICES = RS_LSE_BLK / RS_ROWS;                        // 32
constexpr int RS_LSE_PER = HC_RESCORE_MAX_BLOCKS / RS_LSE_SLICES;          // partials per thread: 16
template <int G>
__global__ __launch_bounds__(RS_LSE_BLK) void rescore_lse_kernel(RescoreBatch batch)
{
    const RescoreArgs& a = batch.it[blockIdx.y];
    if ((int)blockIdx.x >= a.n_reps) return;
    __shared__ float sm_m[RS_LSE_SLICES][RS_ROWS], sm_z[RS_LSE_SLICES][RS_ROWS];
    const int rep = blockIdx.x;
    const RepDev rd = a.reps[rep];
    const int row = threadIdx.x % RS_ROWS, slice = threadIdx.x / RS_ROWS;
    float pm[RS_LSE_PER], pz[RS_LSE_PER];
#pragma unroll
    for (int i = 0; i < RS_LSE_PER; ++i) {
        const int b = slice + i * RS_LSE_SLICES;
        float2 v = make_float2(RS_M_INIT, 0.f);
        if (b < a.nblk) v = *reinterpret_cast<const float2*>(a.part + (((size_t)rep * a.nblk + b) * RS_ROWS + row) * 2);
        pm[i] = v.x;
        pz[i] = v.y;
    }
    float mm = pm[0];
#pragma unroll
    for (int i = 1; i < RS_LSE_PER; ++i) mm = fmaxf(mm, pm[i]);
    float zz = 0.f;
#pragma unroll
    for (int i = 0; i < RS_LSE_PER; ++i) zz += pz[i] * __builtin_amdgcn_exp2f(pm[i] - mm);
    sm_m[slice][row] = mm;
    sm_z[slice][row] = zz;
    __syncthreads();
    if (threadIdx.x < RS_ROWS) {
        float M = sm_m[0][row];
#pragma unroll
        for (int k = 1; k < RS_LSE_SLICES; ++k) M = fmaxf(M, sm_m[k][row]);
        float Z = 0.f;
#pragma unroll
        for (int k = 0; k < RS_LSE_SLICES; ++k) Z += sm_z[k][row] * __builtin_amdgcn_exp2f(sm_m[k][row] - M);
        const int item = row / G, g = row % G;
        if (item < a.n_items) a.lse[(size_t)item * a.lse_item_stride + (size_t)rd.bh * G + g] = (M + __builtin_amdgcn_logf(Z)) * RS_LN2;
    }
}

// The current queries of up to HC_MAX_GROUP layers go into their window buffers with one launch.
struct PushBatch {
    const uint4* src[HC_MAX_GROUP];
    uint4* dst[HC_MAX_GROUP];
    int n16;
};
__global__ __launch_bounds__(RS_BLK) void rescore_push_kernel(PushBatch B)
{
    const uint4* __restrict__ s = B.src[blockIdx.y];
    uint4* __restrict__ d = B.dst[blockIdx.y];
    for (int i = blockIdx.x * RS_BLK + threadIdx.x; i < B.n16; i += gridDim.x * RS_BLK) d[i] = s[i];
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}   // namespace

int hc_rescore_items_per_pass(const hc_ctx* ctx) { return std::min((int)HC_MAX_GROUP, RS_ROWS / ctx->G); }

hc_rescore_layout hc_rescore_plan(const hc_ctx* ctx, const hc_layer* L)
{
    const hc_config& c = ctx->cfg;
    const size_t ni = (size_t)hc_rescore_items_per_pass(ctx);
    hc_rescore_layout o{};
    o.logits_item = (size_t)L->n_reps * c.max_ctx * ctx->G;
    o.scores_item = (size_t)L->n_reps * c.max_ctx;
    o.lse_item = (size_t)c.B * c.Hq;
    o.topk_item = (size_t)c.B * c.Hkv * c.max_k;
    size_t off = 0;
    o.logits_off = off;
    off += align256(ni * o.logits_item * 4);
    o.scores_off = off;
    off += align256(ni * o.scores_item * 4);
    o.lse_off = off;
    off += align256(ni * o.lse_item * 4);
    o.topk_off = off;
    off += align256(ni * o.topk_item * 4);
    o.part_off = off;
    off += align256((size_t)std::max(1, L->n_reps) * HC_RESCORE_MAX_BLOCKS * RS_ROWS * 2 * 4);
    o.scratch_off = off;                 // inter / flag rows the selection passes want to write
    off += align256(2 * (size_t)c.B * c.Hkv * 4);
    o.bytes = off;
    return o;
}

hc_status hc_launch_rescore_push(hc_ctx* ctx, int n, const void* const* q, void* const* dst, hipStream_t st)
{
    if (n < 1 || n > HC_MAX_GROUP) return hc_fail(ctx, HC_EINVAL, "query push of %d layers", n);
    PushBatch B{};
    for (int i = 0; i < n; ++i) {
        B.src[i] = (const uint4*)q[i];
        B.dst[i] = (uint4*)dst[i];
    }
    B.n16 = ctx->cfg.B * ctx->cfg.Hq * HC_D * 2 / 16;
    rescore_push_kernel<<<dim3(std::max(1, std::min(8, B.n16 / RS_BLK)), n), dim3(RS_BLK), 0, st>>>(B);
    HC_HIP(ctx, hipGetLastError());
    return HC_OK;
}

// Logits [n_items][n_heads][max_ctx][G] and lse [n_items][B*Hq] of n_items queries (q, item stride B*Hq*D)
// against the K rows of the heads listed in `reps`: in the arena (src == nullptr: pivots, hd.k_off, hd.len
// rows) or in a prefill buffer (`arena` is that buffer, src[bh].k_off, hd.ctx rows).  One launch for all jobs.
hc_status hc_launch_logits_lse(hc_ctx* ctx, int n_jobs, const hc_logits_job* jobs, int n_items, hipStream_t st)
{
    if (n_items < 1 || n_items > hc_rescore_items_per_pass(ctx)) return hc_fail(ctx, HC_EINVAL, "scoring pass of %d queries", n_items);
    if (n_jobs < 1 || n_jobs > HC_MAX_GROUP) return hc_fail(ctx, HC_EINVAL, "scoring pass over %d layers", n_jobs);
    int total_heads = 0, max_heads = 0, max_len = 1;
    for (int j = 0; j < n_jobs; ++j) {
        total_heads += jobs[j].n_heads;
        max_heads = std::max(max_heads, jobs[j].n_heads);
        max_len = std::max(max_len, jobs[j].max_len);
    }
    if (total_heads == 0) return HC_OK;
    const int tiles = (max_len + RS_WG_TILE - 1) / RS_WG_TILE;
    // two workgroups per compute unit over all heads (measured at 224K, two pivots: 29.5 us, against 33-35 us with
    // three or four and 31 us with one), each with at least two iterations
    const int want = std::max(1, 2 * ctx->n_cu / total_heads);
    const int nblk = std::max(1, std::min({(int)HC_RESCORE_MAX_BLOCKS, want, (tiles + 1) / 2}));
    RescoreBatch B{};
    for (int j = 0; j < n_jobs; ++j) {
        RescoreArgs& a = B.it[j];
        const hc_logits_job& x = jobs[j];
        a.heads = x.L->heads;
        a.reps = x.reps;
        a.arena = (const uint16_t*)x.arena;
        a.q_item_stride = (size_t)ctx->cfg.B * ctx->cfg.Hq * HC_D;
        a.q_first = (const uint16_t*)x.q;
        a.logits = x.logits;
        a.logits_item_stride = x.logits_item;
        a.lse = x.lse;
        a.lse_item_stride = x.lse_item;
        a.part = x.part;
        a.src = x.src;
        a.n_items = n_items;
        a.n_reps = x.n_heads;
        a.max_ctx = ctx->cfg.max_ctx;
        a.nblk = nblk;
    }
    const dim3 grid(nblk, max_heads, n_jobs);
    switch (ctx->G) {
    case 1: rescore_logits_kernel<1><<<grid, dim3(RS_BLK), 0, st>>>(B); break;
    case 2: rescore_logits_kernel<2><<<grid, dim3(RS_BLK), 0, st>>>(B); break;
    case 4: rescore_logits_kernel<4><<<grid, dim3(RS_BLK), 0, st>>>(B); break;
    default: rescore_logits_kernel<8><<<grid, dim3(RS_BLK), 0, st>>>(B); break;
    }
    HC_HIP(ctx, hipGetLastError());
    const dim3 grid2(max_heads, n_jobs);
    switch (ctx->G) {
    case 1: rescore_lse_kernel<1><<<grid2, dim3(RS_LSE_BLK), 0, st>>>(B); break;
    case 2: rescore_lse_kernel<2><<<grid2, dim3(RS_LSE_BLK), 0, st>>>(B); break;
    case 4: rescore_lse_kernel<4><<<grid2, dim3(RS_LSE_BLK), 0, st>>>(B); break;
    default: rescore_lse_kernel<8><<<grid2, dim3(RS_LSE_BLK), 0, st>>>(B); break;
    }
    HC_HIP(ctx, hipGetLastError());
    return HC_OK;
}

// The job of a layer's pivots against buffered queries [first, ...) of its window.
hc_logits_job hc_rescore_job(const hc_ctx* ctx, const hc_layer* L, const void* arena, const void* q_window, int first, void* work)
{
    const hc_rescore_layout lay = hc_rescore_plan(ctx, L);
    int max_len = 1;
    for (size_t i = 0; i < L->hd_host.size(); ++i)
        if (L->rep_slot_of[i] >= 0) max_len = std::max(max_len, (int)L->hd_host[i].len);
    const size_t q_item = (size_t)ctx->cfg.B * ctx->cfg.Hq * HC_D;
    return hc_logits_job{L, L->reps, L->n_reps, max_len, arena, nullptr, (const uint16_t*)q_window + (size_t)first * q_item,
                         (float*)((char*)work + lay.logits_off), lay.logits_item, (float*)((char*)work + lay.lse_off), lay.lse_item,
                         (float*)((char*)work + lay.part_off)};
}
