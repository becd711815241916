// hc_append.hip -- the cache update of ModelForward (Algorithm 1): the decode token's K/V rows enter the
// heterogeneous cache at position ctx of their sequence.
//
// One workgroup of 64 threads per KV head (a row is 256 bytes: 4 bytes per thread).  A full head gets the
// row at the end of its K and V blocks; a compressed head in the slot of its ring of recent positions that
// held the position which now leaves the window; a satellite also in its host-tier block, written over the
// host link, so that the position can be retrieved later.  The same workgroup then moves the lengths in the
// device tables on (the head's context length; a full head's resident length and the end of its last
// split-K segment, in the segment table and in the workgroup descriptor that carries a copy of it; a pivot's
// candidate range), so that no host copy is needed per token.
#include <algorithm>

#include "hc_internal.h"

namespace {

// One layer of a batched call (blockIdx.y picks the layer): the layers of a hc_decode_step group take their
// tokens with one launch.
struct AppendItem {
    HeadDev* heads;
    SegDev* segs;
    BlkDev* blks;
    RepDev* reps;
    const uint32_t* k_new;
    const uint32_t* v_new;
    uint32_t* arena;
    uint32_t* tier;
    int n_heads, pad;
};
struct AppendBatch {
    AppendItem it[HC_MAX_GROUP];
};

__global__ __launch_bounds__(64) void append_kernel(AppendBatch B)
{
    const AppendItem& it = B.it[blockIdx.y];
    if ((int)blockIdx.x >= it.n_heads) return;
    HeadDev* __restrict__ heads = it.heads;
    SegDev* __restrict__ segs = it.segs;
    BlkDev* __restrict__ blks = it.blks;
    RepDev* __restrict__ reps = it.reps;
    const uint32_t* __restrict__ k_new = it.k_new;
    const uint32_t* __restrict__ v_new = it.v_new;
    uint32_t* __restrict__ arena = it.arena;
    uint32_t* __restrict__ tier = it.tier;
    const int bh = blockIdx.x, t = threadIdx.x;
    const HeadDev hd = heads[bh];
    const int pos = hd.ctx;                                      // the new position
    const uint32_t kw = k_new[(size_t)bh * (HC_D / 2) + t], vw = v_new[(size_t)bh * (HC_D / 2) + t];
    int slot = -1;
    if (hd.role == HC_ROLE_FULL) {
        slot = pos;
    } else if (hd.recent > 0) {
        slot = hd.sink + (pos - hd.ctx0) % hd.recent;            // pos >= ctx0: the slot of position pos - recent
    }
    if (slot >= 0) {
        arena[(hd.k_off + (int64_t)slot * HC_D) / 2 + t] = kw;   // offsets are multiples of 8 elements
        arena[(hd.v_off + (int64_t)slot * HC_D) / 2 + t] = vw;
    }
    if (hd.role == HC_ROLE_SATELLITE) {
        uint32_t* row = tier + (hd.tier_off + (int64_t)pos * 2 * HC_D) / 2;
        row[t] = kw;
        row[HC_D / 2 + t] = vw;
    }
    __syncthreads();                                             // everyone has read the old table entry
    if (t == 0) {
        heads[bh].ctx = pos + 1;
        if (hd.role == HC_ROLE_FULL) {
            heads[bh].len = hd.len + 1;
            if (hd.tail_seg >= 0) segs[hd.tail_seg].row_end = hd.len + 1;
            if (hd.tail_blk >= 0) blks[hd.tail_blk].first.row_end = hd.len + 1;
            if (hd.rep_slot >= 0) {
                RepDev* r = reps + hd.rep_slot;
                const int hi = r->hi + 1;
                r->hi = hi;
                r->nchunk = (hi - r->lo + HC_SEL_CHUNK - 1) / HC_SEL_CHUNK;
            }
        }
    }
}

}   // namespace

hc_status hc_launch_append(hc_ctx* ctx, int n, const hc_append_call* calls, hipStream_t st)
{
    if (n < 1 || n > HC_MAX_GROUP) return hc_fail(ctx, HC_EINVAL, "append batch of %d layers", n);
    AppendBatch B{};
    int max_heads = 0;
    for (int i = 0; i < n; ++i) {
        const hc_append_call& x = calls[i];
        B.it[i] = AppendItem{x.L->heads, x.L->segs, x.L->blks, x.L->reps, (const uint32_t*)x.k_new, (const uint32_t*)x.v_new,
                             (uint32_t*)x.arena, (uint32_t*)x.tier, x.L->n_heads, 0};
        max_heads = std::max(max_heads, x.L->n_heads);
    }
    append_kernel<<<dim3(max_heads, n), dim3(64), 0, st>>>(B);
    HC_HIP(ctx, hipGetLastError());
    return HC_OK;
}
