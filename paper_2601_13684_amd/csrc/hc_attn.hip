// hc_attn.hip -- decode attention over the heterogeneous KV cache (Algorithm 1, ModelForward over
// C_GPU; resident sets of Sec. 4.3), written for CDNA4 (gfx950, 64-wide wavefronts).
//
// The work is GEMV-shaped and HBM-bound: every K/V byte is used once, by one lane.  So K and V
// rows stream straight from HBM into registers with 16-byte coalesced loads (no LDS staging: there
// is no reuse a shared tile could serve), and the arithmetic is plain VALU: packed-bf16 dot
// products (v_dot2c_f32_bf16) for q.K and fp32 FMAs for p.V.
//
// Lane layout of one wavefront: 8 rows x 8 column lanes.  Lane (r, c) loads 16-byte chunks c and
// c+8 of row r, i.e. elements [8c, 8c+8) and [64+8c, 64+8c+8): each load instruction reads eight
// complete 128-byte lines.  The same lane owns the same row of V, so the softmax weight it
// computes (after a 3-step DPP all-reduce over the 8 column lanes) is already where p.V needs it.
//
// The running maximum is kept wave-uniform and updated lazily (only when some logit exceeds it by
// more than 2^16): partial sums of different lanes then share one reference and merge by plain
// addition.  A workgroup (4 wavefronts) owns a contiguous share of the layer's rows (split-K over
// ragged per-head lengths) and writes one partial (max, sum, acc[G][D]) per head it touches; a
// second kernel combines the partials.
#include "hc_internal.h"

namespace {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}

// Cross-lane moves inside a row of 16 lanes (data-parallel primitives, no LDS traffic).
template <int CTRL>
__device__ __forceinline__ float dpp(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}
constexpr int DPP_XOR1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141; // lane i <-> 7-i inside each group of 8
constexpr int DPP_ROR8 = 0x128;        // lane i <-> i^8 inside a row of 16

__device__ __forceinline__ float sum8(float x)   // sum over the 8 column lanes, result in all of them
{
    x += dpp<DPP_XOR1>(x);
    x += dpp<DPP_XOR2>(x);
    x += dpp<DPP_HALF_MIRROR>(x);
    return x;
}

__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float LAZY_SLACK = 16.0f;     // log2 units: exp2 of at most 2^16 before the reference moves
constexpr float M_INIT = -1.0e30f;      // finite, so that (old - new) never is inf - inf

template <int G>
struct WaveState {
    float m[G];          // reference maximum, log2 units, identical in all lanes
    float Z[G];          // sum of exp2(t - m) over the rows this lane handled
    float acc[G][16];    // sum of exp2(t - m) * V[row][d] for the lane's 16 columns
};

// One row step: the wave's 8 rows [row0, row0+8).  k0,k1 / v0,v1 are the lane's two 16-byte chunks.
template <int G, bool MASKED>
__device__ __forceinline__ void row_step(WaveState<G>& st, const uint32_t (&qreg)[G][8], const uint4& k0,
                                         const uint4& k1, const uint4& v0, const uint4& v1, bool valid,
                                         float* __restrict__ rep_row, int max_ctx, int c)
{
    float s[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float a = 0.f;
        a = dot2(k0.x, qreg[g][0], a);
        a = dot2(k0.y, qreg[g][1], a);
        a = dot2(k0.z, qreg[g][2], a);
        a = dot2(k0.w, qreg[g][3], a);
        a = dot2(k1.x, qreg[g][4], a);
        a = dot2(k1.y, qreg[g][5], a);
        a = dot2(k1.z, qreg[g][6], a);
        a = dot2(k1.w, qreg[g][7], a);
        s[g] = sum8(a);
    }
    if (rep_row) {   // pivot head: keep the scaled logits for the drift monitor
        float mine = s[0];
#pragma unroll
        for (int g = 1; g < G; ++g) mine = (c == g) ? s[g] : mine;
        if (c < G && (!MASKED || valid)) rep_row[(size_t)c * max_ctx] = mine * 0.08838834764831845f;   // 1/sqrt(128)
    }
    float t[G];
    bool over = false;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        t[g] = s[g] * (LOG2E * 0.08838834764831845f);
        if (MASKED && !valid) t[g] = -INFINITY;
        over |= t[g] > st.m[g] + LAZY_SLACK;
    }
    if (__builtin_amdgcn_ballot_w64(over) != 0) {   // rare: move the reference maximum
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float x = t[g];
            x = fmaxf(x, dpp<DPP_ROR8>(x));
            x = fmaxf(x, __shfl_xor(x, 16));
            x = fmaxf(x, __shfl_xor(x, 32));
            const float mn = fmaxf(st.m[g], x);
            const float alpha = __builtin_amdgcn_exp2f(st.m[g] - mn);
            st.m[g] = mn;
            st.Z[g] *= alpha;
#pragma unroll
            for (int i = 0; i < 16; ++i) st.acc[g][i] *= alpha;
        }
    }
    float vf[16];
    vf[0] = bf_lo(v0.x); vf[1] = bf_hi(v0.x); vf[2] = bf_lo(v0.y); vf[3] = bf_hi(v0.y);
    vf[4] = bf_lo(v0.z); vf[5] = bf_hi(v0.z); vf[6] = bf_lo(v0.w); vf[7] = bf_hi(v0.w);
    vf[8] = bf_lo(v1.x); vf[9] = bf_hi(v1.x); vf[10] = bf_lo(v1.y); vf[11] = bf_hi(v1.y);
    vf[12] = bf_lo(v1.z); vf[13] = bf_hi(v1.z); vf[14] = bf_lo(v1.w); vf[15] = bf_hi(v1.w);
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float p = __builtin_amdgcn_exp2f(t[g] - st.m[g]);
        st.Z[g] += p;
#pragma unroll
        for (int i = 0; i < 16; ++i) st.acc[g][i] = fmaf(p, vf[i], st.acc[g][i]);
    }
}

template <int G, int U, int WG_PER_CU>
__global__ __launch_bounds__(256, WG_PER_CU) void attn_split_kernel(const uint16_t* __restrict__ arena,
                                                            const uint16_t* __restrict__ q,
                                                            const HeadDev* __restrict__ heads,
                                                            const SegDev* __restrict__ segs,
                                                            const int32_t* __restrict__ blk_seg,
                                                            float* __restrict__ part_acc, float* __restrict__ part_ml,
                                                            float* __restrict__ rep_logits, int max_ctx)
{
    __shared__ float sm_m[4][G];
    __shared__ float sm_Z[8][G];
    __shared__ float sm_red[8][G * HC_D];

    const int tid = threadIdx.x;
    const int w = tid >> 6;
    const int lane = tid & 63;
    const int r = lane >> 3;     // row inside a row step
    const int c = lane & 7;      // column lane

    const int seg_end = blk_seg[blockIdx.x + 1];
    for (int si = blk_seg[blockIdx.x]; si < seg_end; ++si) {
        const SegDev seg = segs[si];
        const HeadDev hd = heads[seg.bh];
        const uint16_t* __restrict__ Kp = arena + hd.k_off;
        const uint16_t* __restrict__ Vp = arena + hd.v_off;
        float* rep_base = (rep_logits && hd.rep_slot >= 0) ? rep_logits + (size_t)hd.rep_slot * G * max_ctx : nullptr;

        uint32_t qreg[G][8];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint4* qp = reinterpret_cast<const uint4*>(q + ((size_t)seg.bh * G + g) * HC_D);
            const uint4 a = qp[c], b = qp[8 + c];
            qreg[g][0] = a.x; qreg[g][1] = a.y; qreg[g][2] = a.z; qreg[g][3] = a.w;
            qreg[g][4] = b.x; qreg[g][5] = b.y; qreg[g][6] = b.z; qreg[g][7] = b.w;
        }
        WaveState<G> st;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            st.m[g] = M_INIT;
            st.Z[g] = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) st.acc[g][i] = 0.f;
        }

        // Row steps of this wave: rows seg.row_begin + 8*(w + 4*i), i = 0, 1, ...
        int row0 = seg.row_begin + 8 * w;
        // full groups of U row steps, no bounds checks
        for (; row0 + 32 * (U - 1) + 8 <= seg.row_end; row0 += 32 * U) {
            uint4 k0[U], k1[U], v0[U], v1[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const size_t off = (size_t)(row0 + 32 * u + r) * HC_D;
                const uint4* kp = reinterpret_cast<const uint4*>(Kp + off);
                const uint4* vp = reinterpret_cast<const uint4*>(Vp + off);
                k0[u] = kp[c];
                k1[u] = kp[8 + c];
                v0[u] = vp[c];
                v1[u] = vp[8 + c];
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                row_step<G, false>(st, qreg, k0[u], k1[u], v0[u], v1[u], true,
                                   rep_base ? rep_base + row0 + 32 * u + r : nullptr, max_ctx, c);
        }
        // remaining row steps one at a time; rows past the end are clamped for the load and masked
        for (; row0 < seg.row_end; row0 += 32) {
            const int row = row0 + r;
            const bool valid = row < seg.row_end;
            const size_t off = (size_t)(valid ? row : seg.row_end - 1) * HC_D;
            const uint4* kp = reinterpret_cast<const uint4*>(Kp + off);
            const uint4* vp = reinterpret_cast<const uint4*>(Vp + off);
            const uint4 k0 = kp[c], k1 = kp[8 + c], v0 = vp[c], v1 = vp[8 + c];
            row_step<G, true>(st, qreg, k0, k1, v0, v1, valid, rep_base ? rep_base + row : nullptr, max_ctx, c);
        }

        // ---- merge the 4 waves x 8 row lanes into one partial (4 row lanes in registers, the rest in LDS) ----
        if (lane == 0) {
#pragma unroll
            for (int g = 0; g < G; ++g) sm_m[w][g] = st.m[g];
        }
        __syncthreads();
        float M[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            M[g] = fmaxf(fmaxf(sm_m[0][g], sm_m[1][g]), fmaxf(sm_m[2][g], sm_m[3][g]));
            const float sc = __builtin_amdgcn_exp2f(st.m[g] - M[g]);
            float z = st.Z[g] * sc;
            z += dpp<DPP_ROR8>(z);
            z += __shfl_xor(z, 16);
            if ((lane & 31) == 0) sm_Z[w * 2 + (lane >> 5)][g] = z;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float a = st.acc[g][i] * sc;
                a += dpp<DPP_ROR8>(a);
                a += __shfl_xor(a, 16);
                st.acc[g][i] = a;
            }
        }
        if ((lane & 24) == 0) {
            float* dst = sm_red[w * 2 + (lane >> 5)];
#pragma unroll
            for (int g = 0; g < G; ++g) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    dst[g * HC_D + 8 * c + i] = st.acc[g][i];
                    dst[g * HC_D + 64 + 8 * c + i] = st.acc[g][8 + i];
                }
            }
        }
        __syncthreads();
        for (int o = tid; o < G * HC_D; o += 256) {
            float a = 0.f;
#pragma unroll
            for (int p = 0; p < 8; ++p) a += sm_red[p][o];
            part_acc[(size_t)seg.slot * G * HC_D + o] = a;
        }
        if (tid < G) {
            float z = 0.f;
#pragma unroll
            for (int p = 0; p < 8; ++p) z += sm_Z[p][tid];
            part_ml[((size_t)seg.slot * G + tid) * 2 + 0] = M[tid];
            part_ml[((size_t)seg.slot * G + tid) * 2 + 1] = z;
        }
        __syncthreads();
    }
}

// Second pass: out = sum_s 2^(m_s - M) acc_s / sum_s 2^(m_s - M) Z_s over the partials of one head.
// One workgroup of 1024 threads per (b, query head): 8 partial lanes x 128 columns.
template <int G>
__global__ __launch_bounds__(1024) void attn_combine_kernel(const HeadDev* __restrict__ heads,
                                                            const float* __restrict__ part_acc,
                                                            const float* __restrict__ part_ml,
                                                            float* __restrict__ out, float* __restrict__ lse)
{
    __shared__ float sm_max[16];
    __shared__ float sm_acc[8][HC_D];
    __shared__ float sm_z[8];
    const int bh = blockIdx.x / G, g = blockIdx.x % G;
    const HeadDev hd = heads[bh];
    const int tid = threadIdx.x, d = tid & 127, pl = tid >> 7;
    const int n = hd.part_count;

    float mx = M_INIT;
    for (int s = tid; s < n; s += 1024) mx = fmaxf(mx, part_ml[((size_t)(hd.part_begin + s) * G + g) * 2]);
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if ((tid & 63) == 0) sm_max[tid >> 6] = mx;
    __syncthreads();
    float M = sm_max[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) M = fmaxf(M, sm_max[i]);

    float acc = 0.f, z = 0.f;
    for (int s = pl; s < n; s += 8) {
        const size_t slot = (size_t)(hd.part_begin + s);
        const float wgt = __builtin_amdgcn_exp2f(part_ml[(slot * G + g) * 2] - M);
        z += wgt * part_ml[(slot * G + g) * 2 + 1];
        acc += wgt * part_acc[(slot * G + g) * HC_D + d];
    }
    sm_acc[pl][d] = acc;
    if (d == 0) sm_z[pl] = z;
    __syncthreads();
    if (pl == 0) {
        float a = 0.f, zz = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a += sm_acc[i][d];
            zz += sm_z[i];
        }
        out[(size_t)blockIdx.x * HC_D + d] = a / zz;
        if (d == 0) lse[blockIdx.x] = (M + __builtin_amdgcn_logf(zz)) * LN2;
    }
}

// Rows in flight per wave (U row steps of 8 rows, 4 KB each) against registers: the group-of-4 case
// holds 32 query + 64 accumulator registers and takes U = 4 at two workgroups per compute unit.
template <int G> struct Tune { static constexpr int U = 4, WG = 2; };
template <> struct Tune<8> { static constexpr int U = 1, WG = 2; };

template <int G>
hc_status launch(hc_ctx* ctx, const hc_layer* L, const void* arena, const void* q, float* out, float* lse,
                 float* rep_logits, hipStream_t st)
{
    attn_split_kernel<G, Tune<G>::U, Tune<G>::WG><<<dim3(L->n_blocks), dim3(256), 0, st>>>(
        (const uint16_t*)arena, (const uint16_t*)q, L->heads, L->segs, L->blk_seg, ctx->part_acc, ctx->part_ml,
        rep_logits, ctx->cfg.max_ctx);
    HC_HIP(ctx, hipGetLastError());
    attn_combine_kernel<G><<<dim3(L->n_heads * G), dim3(1024), 0, st>>>(L->heads, ctx->part_acc, ctx->part_ml, out, lse);
    HC_HIP(ctx, hipGetLastError());
    return HC_OK;
}

}   // namespace

hc_status hc_launch_attn(hc_ctx* ctx, const hc_layer* L, const void* arena, const void* q, float* out, float* lse,
                         float* rep_logits, hipStream_t st)
{
    if ((size_t)L->n_partials > ctx->part_slots) return hc_fail(ctx, HC_ESTATE, "split-K workspace smaller than the plan");
    switch (ctx->G) {
    case 1: return launch<1>(ctx, L, arena, q, out, lse, rep_logits, st);
    case 2: return launch<2>(ctx, L, arena, q, out, lse, rep_logits, st);
    case 4: return launch<4>(ctx, L, arena, q, out, lse, rep_logits, st);
    case 8: return launch<8>(ctx, L, arena, q, out, lse, rep_logits, st);
    }
    return hc_fail(ctx, HC_ESHAPE, "unsupported group size");
}
