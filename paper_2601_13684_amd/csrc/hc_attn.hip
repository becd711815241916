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
// more than 2^16, which leaves the streaming loop): partial sums of different lanes then share one
// reference and merge by plain addition.  A workgroup (4 wavefronts) owns a contiguous share of the layer's rows (split-K over
// ragged per-head lengths) and writes one partial (max, sum, acc[G][D]) per head it touches; a
// second kernel combines the partials.  Loads are double-buffered in registers: the next group of
// row steps is in flight while the current one is being reduced.
#include <hip/hip_ext.h>

#include <algorithm>

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

// Lane-swap instructions of gfx950.  swap_rows16: the odd rows of 16 lanes of x change places with the even
// rows of y (x becomes [x.row0, y.row0, x.row2, y.row2], y becomes [x.row1, y.row1, x.row3, y.row3]);
// swap_halves32: the upper 32 lanes of x change places with the lower 32 lanes of y.  Written as assembly
// because the compiler folds "first result + second result" of the corresponding builtins into twice the
// first (checked on ROCm 7.2); the s_nop covers the wait states the instruction needs after a vector write
// of its operands.
__device__ __forceinline__ void swap_rows16(float& x, float& y)
{
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(x), "+v"(y));
}
__device__ __forceinline__ void swap_halves32(float& x, float& y)
{
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(x), "+v"(y));
}

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
constexpr float INV_SQRT_D = 0.08838834764831845f;   // 1/sqrt(128)
constexpr float LAZY_SLACK = 16.0f;     // log2 units: exp2 of at most 2^16 before the reference moves
constexpr float M_INIT = -1.0e30f;      // finite, so that (old - new) never is inf - inf

template <int G>
struct WaveState {
    float m[G];          // reference maximum, log2 units, identical in all lanes
    float Z[G];          // sum of exp2(t - m) over the rows this lane handled
    float acc[G][16];    // sum of exp2(t - m) * V[row][d] for the lane's 16 columns
};

// The pivot-logit filter of the segment being streamed (all fields wave-uniform).  A pivot's scaled logits are
// what the drift monitor scores; with the filter on only the rows that can matter to it are kept: row j stays if
// sum_g 2^(t_g[j] - ref_g) >= cutsum, where ref is the log-sum-exp the monitor saw at the step that set the filter
// and cutsum a fraction of the smallest score that made it into a list then.  The monitor checks afterwards, with
// this step's own log-sum-exp, that no dropped row could have reached a list, and otherwise has every logit
// computed again; so the filter changes what is written, never what is selected.  (A cheaper test on the largest
// of the four exponents alone keeps several times as many rows when the heads of a group attend differently.)
template <int G>
struct FilterCtx {
    float cutsum;
    float ref[G];       // log2 units
    int lo, hi;         // the pivot's candidate positions
};

// One row step of a wave (its 8 rows): the lane's two 16-byte chunks of its K row and of its V row.
struct Tile {
    uint4 k0, k1, v0, v1;
};

// Kb / Vb: the head's K and V blocks (wave-uniform byte pointers); off: the lane's byte offset of its
// first chunk (row * 256 + c * 16, below 4 GiB because contexts are capped at 2^24 rows).
__device__ __forceinline__ void load_tile(Tile& t, const char* __restrict__ Kb, const char* __restrict__ Vb, uint32_t off)
{
    // K/V rows are read once per pass: streaming (non-temporal) loads keep them from displacing what the
    // caches are useful for here, and measured 9 % faster than plain loads at the 224K shape.
    typedef uint32_t u4v __attribute__((ext_vector_type(4)));
    const u4v k0 = __builtin_nontemporal_load(reinterpret_cast<const u4v*>(Kb + off));
    const u4v k1 = __builtin_nontemporal_load(reinterpret_cast<const u4v*>(Kb + off + 128));
    const u4v v0 = __builtin_nontemporal_load(reinterpret_cast<const u4v*>(Vb + off));
    const u4v v1 = __builtin_nontemporal_load(reinterpret_cast<const u4v*>(Vb + off + 128));
    t.k0 = make_uint4(k0.x, k0.y, k0.z, k0.w);
    t.k1 = make_uint4(k1.x, k1.y, k1.z, k1.w);
    t.v0 = make_uint4(v0.x, v0.y, v0.z, v0.w);
    t.v1 = make_uint4(v1.x, v1.y, v1.z, v1.w);
}

// q.K of the lane's row for the G query heads: partial dot products over the lane's 16 columns,
// then summed over the 8 column lanes (every lane of the row ends up with the full sums).
template <int G>
__device__ __forceinline__ void qk(const uint32_t (&qreg)[G][8], const Tile& t, float (&s)[G])
{
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float a = 0.f;
        a = dot2(t.k0.x, qreg[g][0], a);
        a = dot2(t.k0.y, qreg[g][1], a);
        a = dot2(t.k0.z, qreg[g][2], a);
        a = dot2(t.k0.w, qreg[g][3], a);
        a = dot2(t.k1.x, qreg[g][4], a);
        a = dot2(t.k1.y, qreg[g][5], a);
        a = dot2(t.k1.z, qreg[g][6], a);
        a = dot2(t.k1.w, qreg[g][7], a);
        s[g] = sum8(a);
    }
}

// The G scaled logits of the lane's row, kept for the drift monitor.  Only column lane 0 holds them after
// the reduction.  They go to a staging buffer in LDS first (stash points at the row's G floats there) and
// reach memory in long contiguous runs: 128-byte stores scattered through a pass that streams reads at
// full rate cost several times their share of the traffic.
template <int G>
__device__ __forceinline__ void stash_rep(float* stash, const float (&s)[G], int c, bool valid)
{
    if (c != 0 || !valid) return;
    const float first = s[0] * INV_SQRT_D;
    if (G == 1) {
        stash[0] = first;
    } else if (G == 2) {
        *reinterpret_cast<float2*>(stash) = make_float2(first, s[1] * INV_SQRT_D);
    } else {
        reinterpret_cast<float4*>(stash)[0] = make_float4(first, s[1] * INV_SQRT_D, s[2] * INV_SQRT_D, s[3] * INV_SQRT_D);
#pragma unroll
        for (int q = 1; q < G / 4; ++q)
            reinterpret_cast<float4*>(stash)[q] = make_float4(s[4 * q] * INV_SQRT_D, s[4 * q + 1] * INV_SQRT_D,
                                                              s[4 * q + 2] * INV_SQRT_D, s[4 * q + 3] * INV_SQRT_D);
    }
}

// Exponents of the softmax weights relative to the reference, x[g] = log2(e)/sqrt(D) s[g] - m[g]
// (-inf for a masked row).  Returns the wave's mask of lanes in which some exponent exceeds the slack:
// non-zero means the reference has to move before this row step may be accumulated.
template <int G>
__device__ __forceinline__ uint64_t exponents(const WaveState<G>& st, const float (&s)[G], float (&x)[G], bool valid)
{
    float mx = -INFINITY;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        x[g] = valid ? fmaf(s[g], LOG2E * INV_SQRT_D, -st.m[g]) : -INFINITY;
        mx = fmaxf(mx, x[g]);
    }
    return __builtin_amdgcn_ballot_w64(mx > LAZY_SLACK);
}

// Rare: raise the reference to the largest logit of this row step and recompute the exponents.
// Returns, per head, the factor 2^(old reference - new reference) by which everything accumulated so
// far has to be multiplied.
template <int G>
__device__ __forceinline__ void move_reference(WaveState<G>& st, const float (&s)[G], float (&x)[G], float (&alpha)[G], bool valid)
{
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float t = valid ? s[g] * (LOG2E * INV_SQRT_D) : -INFINITY;
        float hi = t;
        hi = fmaxf(hi, dpp<DPP_ROR8>(hi));
        hi = fmaxf(hi, __shfl_xor(hi, 16));
        hi = fmaxf(hi, __shfl_xor(hi, 32));
        const float mn = fmaxf(st.m[g], hi);
        alpha[g] = __builtin_amdgcn_exp2f(st.m[g] - mn);
        st.m[g] = mn;
        x[g] = t - mn;
    }
}

// Multiplies the accumulators of one head by alpha if (and only if) the wave-uniform mask is non-zero.
// Written as one opaque block with tied operands so that the accumulators keep their registers on both
// paths: expressed as an ordinary branch, the register allocator copies all of them on the common path.
__device__ __forceinline__ void scale_if(uint64_t mask, float alpha, float& z, float (&a)[16])
{
    asm volatile(
        "s_cmp_eq_u64 %[m], 0\n\t"
        "s_cbranch_scc1 1f\n\t"
        "v_mul_f32 %[z], %[al], %[z]\n\t"
        "v_mul_f32 %[a0], %[al], %[a0]\n\t"
        "v_mul_f32 %[a1], %[al], %[a1]\n\t"
        "v_mul_f32 %[a2], %[al], %[a2]\n\t"
        "v_mul_f32 %[a3], %[al], %[a3]\n\t"
        "v_mul_f32 %[a4], %[al], %[a4]\n\t"
        "v_mul_f32 %[a5], %[al], %[a5]\n\t"
        "v_mul_f32 %[a6], %[al], %[a6]\n\t"
        "v_mul_f32 %[a7], %[al], %[a7]\n\t"
        "v_mul_f32 %[a8], %[al], %[a8]\n\t"
        "v_mul_f32 %[a9], %[al], %[a9]\n\t"
        "v_mul_f32 %[a10], %[al], %[a10]\n\t"
        "v_mul_f32 %[a11], %[al], %[a11]\n\t"
        "v_mul_f32 %[a12], %[al], %[a12]\n\t"
        "v_mul_f32 %[a13], %[al], %[a13]\n\t"
        "v_mul_f32 %[a14], %[al], %[a14]\n\t"
        "v_mul_f32 %[a15], %[al], %[a15]\n"
        "1:"
        : [z] "+v"(z), [a0] "+v"(a[0]), [a1] "+v"(a[1]), [a2] "+v"(a[2]), [a3] "+v"(a[3]), [a4] "+v"(a[4]),
          [a5] "+v"(a[5]), [a6] "+v"(a[6]), [a7] "+v"(a[7]), [a8] "+v"(a[8]), [a9] "+v"(a[9]), [a10] "+v"(a[10]),
          [a11] "+v"(a[11]), [a12] "+v"(a[12]), [a13] "+v"(a[13]), [a14] "+v"(a[14]), [a15] "+v"(a[15])
        : [m] "s"(mask), [al] "v"(alpha)
        : "scc");
}

// p.V: weights 2^x[g], accumulated into the lane's 16 columns.
template <int G>
__device__ __forceinline__ void pv(WaveState<G>& st, const float (&x)[G], const Tile& t)
{
    float vf[16];
    vf[0] = bf_lo(t.v0.x); vf[1] = bf_hi(t.v0.x); vf[2] = bf_lo(t.v0.y); vf[3] = bf_hi(t.v0.y);
    vf[4] = bf_lo(t.v0.z); vf[5] = bf_hi(t.v0.z); vf[6] = bf_lo(t.v0.w); vf[7] = bf_hi(t.v0.w);
    vf[8] = bf_lo(t.v1.x); vf[9] = bf_hi(t.v1.x); vf[10] = bf_lo(t.v1.y); vf[11] = bf_hi(t.v1.y);
    vf[12] = bf_lo(t.v1.z); vf[13] = bf_hi(t.v1.z); vf[14] = bf_lo(t.v1.w); vf[15] = bf_hi(t.v1.w);
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float p = __builtin_amdgcn_exp2f(x[g]);
        st.Z[g] += p;
#pragma unroll
        for (int i = 0; i < 16; ++i) st.acc[g][i] = fmaf(p, vf[i], st.acc[g][i]);
    }
}

// One row step: logits, (pivot) logit stash, reference check, accumulate.  The row loop is the same with and
// without the pivot-logit filter: which of the staged rows are kept is decided when a chunk is written out.
template <int G>
__device__ __forceinline__ void row_step(WaveState<G>& st, const uint32_t (&qreg)[G][8], const Tile& t, float* stash, int c, bool valid)
{
    float s[G], x[G], alpha[G];
    qk<G>(qreg, t, s);
    if (stash) stash_rep<G>(stash, s, c, valid);
    const uint64_t over = exponents<G>(st, s, x, valid);
#pragma unroll
    for (int g = 0; g < G; ++g) alpha[g] = 1.0f;
    if (over) move_reference<G>(st, s, x, alpha, valid);
#pragma unroll
    for (int g = 0; g < G; ++g) scale_if(over, alpha[g], st.Z[g], st.acc[g]);
    pv<G>(st, x, t);
}

// The filter's statistic of a staged row, sum_g 2^(t_g - ref_g) with t the scaled logit in log2 units, against the
// cut (not "sum >= cut": a statistic that is not a number keeps its row).
template <int G>
__device__ __forceinline__ bool keeps(const float* row, const FilterCtx<G>& fc)
{
    float l[G];
    if (G == 1) l[0] = row[0];
    else if (G == 2) { const float2 t = *reinterpret_cast<const float2*>(row); l[0] = t.x; l[1] = t.y; }
    else {
#pragma unroll
        for (int q = 0; q < G / 4; ++q) {
            const float4 t = reinterpret_cast<const float4*>(row)[q];
            l[4 * q] = t.x; l[4 * q + 1] = t.y; l[4 * q + 2] = t.z; l[4 * q + 3] = t.w;
        }
    }
    float est = 0.f;
#pragma unroll
    for (int g = 0; g < G; ++g) est += __builtin_amdgcn_exp2f(fmaf(l[g], LOG2E, -fc.ref[g]));
    return !(est < fc.cutsum);
}

constexpr int REP_STASH_FLOATS = 4096;   // one staging buffer: 16 KB, i.e. 1024 positions of a group of 4 (measured: the
                                         // longer the runs, the cheaper the stores; two workgroups' buffers still fit a CU's LDS)

// Writes the kept rows of one staged chunk (n positions from `first`, logits in src) to rows at, at + 1, ... of the
// pivot's block of rep_logits and their positions to the same entries of kept_pos; returns how many (the same in
// every thread).  Called by the whole workgroup after a barrier that follows the chunk's last staged row; holds one
// barrier itself.  Every wave takes a quarter of the chunk's positions, 64 at a time in position order: first it
// counts the rows it will keep (candidate positions whose statistic reaches the cut), then, knowing the other
// waves' counts, it writes them.
template <int G>
__device__ __forceinline__ int write_kept(const float* src, int first, int n, float* __restrict__ rep_base, int32_t* __restrict__ kept_pos,
                                          int at, const FilterCtx<G>& fc, int (&sm_cnt)[4], int w, int lane)
{
    constexpr int CAP = REP_STASH_FLOATS / G, Q = CAP / 4, ROUNDS = Q / 64;
    static_assert(Q % 64 == 0, "a wave's quarter of a chunk is whole rounds of 64 positions");
    static_assert(ROUNDS <= 32, "a lane remembers its decisions of a chunk in one word");
    constexpr int UNR = ROUNDS < 4 ? ROUNDS : 4;
    int mine = 0;
    uint32_t kept_bits = 0;              // bit rd: this lane's row of round rd is kept
    // (unrolled: the rounds' LDS reads and exponentials overlap; rows past the chunk's end read staged data of an
    // earlier chunk or nothing that matters, and are masked)
#pragma unroll UNR
    for (int rd = 0; rd < ROUNDS; ++rd) {
        const int j = w * Q + rd * 64 + lane;
        const bool keep = keeps<G>(src + (size_t)j * G, fc) && j < n && first + j >= fc.lo && first + j < fc.hi;
        kept_bits |= keep ? 1u << rd : 0u;
        mine += __builtin_popcountll(__builtin_amdgcn_ballot_w64(keep));
    }
    if (lane == 0) sm_cnt[w] = mine;
    __syncthreads();
    const int c0 = sm_cnt[0], c1 = sm_cnt[1], c2 = sm_cnt[2], c3 = sm_cnt[3];
    at += (w > 0 ? c0 : 0) + (w > 1 ? c1 : 0) + (w > 2 ? c2 : 0);
    if (mine > 0) {
#pragma unroll UNR
        for (int rd = 0; rd < ROUNDS; ++rd) {
            const int j = w * Q + rd * 64 + lane;
            const bool keep = (kept_bits >> rd) & 1u;
            const uint64_t m = __builtin_amdgcn_ballot_w64(keep);
            if (keep) {
                const int idx = at + __builtin_popcountll(m & ((1ull << lane) - 1ull));
                const float* e_l = src + (size_t)j * G;
                float* d = rep_base + (size_t)idx * G;
                typedef float f4v __attribute__((ext_vector_type(4)));
                if (G == 1) d[0] = e_l[0];
                else if (G == 2) *reinterpret_cast<float2*>(d) = *reinterpret_cast<const float2*>(e_l);
                else {
#pragma unroll
                    for (int q4 = 0; q4 < G / 4; ++q4) reinterpret_cast<f4v*>(d)[q4] = reinterpret_cast<const f4v*>(e_l)[q4];
                }
                kept_pos[idx] = first + j;
            }
            at += __builtin_popcountll(m);
        }
    }
    return c0 + c1 + c2 + c3;
}

// Streams rows [row_begin, row_end) of one head through the wave state.  The wave takes the row steps
// row_begin + 8*w + 32*i.  Full row steps are double-buffered in registers (tile B is in flight while
// tile A is reduced, and vice versa); the ragged last row step is clamped for the load and masked.
//
// For a pivot whose logits are stored densely (rep_base != nullptr, !FILT) the rows are taken in chunks of
// REP_STASH_FLOATS / G positions: the waves stash their logits in LDS, and at the end of a chunk the workgroup
// writes the chunk's logits to memory as one contiguous run.  Two staging buffers alternate, so one barrier per
// chunk is enough; the number of chunks depends only on the segment, so every wave reaches every barrier.  The
// register pipeline of loads runs on across chunk boundaries.  With the filter (FILT) a chunk's kept rows, in
// position order, are appended to rows row_begin, row_begin + 1, ... of the pivot's block of rep_logits (a segment
// never keeps more rows than it has) and their positions to the same entries of kept_pos (write_kept); the
// segment's last chunk is left staged for the caller, which writes it out behind the barrier of its merge; the
// number of rows kept of the chunks before it is returned (the same in every thread).
template <int G, bool FILT>
__device__ __forceinline__ int process_rows(WaveState<G>& st, const uint32_t (&qreg)[G][8],
                                            const char* __restrict__ Kb, const char* __restrict__ Vb,
                                            float* __restrict__ rep_base, FilterCtx<G>& fc, int32_t* __restrict__ kept_pos,
                                            float (&stash)[FILT ? 1 : 2][REP_STASH_FLOATS], int (&sm_cnt)[4],
                                            int row_begin, int row_end, int w, int r, int c)
{
    constexpr int CAP = REP_STASH_FLOATS / G;      // positions per chunk
    constexpr int STEPS = CAP / 32;                // row steps of one wave per chunk
    static_assert(STEPS % 2 == 0, "chunks hold whole pairs of row steps");
    constexpr uint32_t STEP = 32u * 256u;          // bytes from one row step of this wave to the next
    const int wave_row0 = row_begin + 8 * w;
    const int nfull = wave_row0 + 8 <= row_end ? (row_end - 8 - wave_row0) / 32 + 1 : 0;   // unmasked row steps
    uint32_t off = (uint32_t)(wave_row0 + r) * 256u + (uint32_t)c * 16u;                   // the lane's first chunk of its row
    const bool dense = rep_base != nullptr;
    int seg_kept = 0;
    const int nchunk = dense ? (row_end - row_begin + CAP - 1) / CAP : 1;
    Tile A, B;
    int i = 0;
    if (nfull > 0) load_tile(A, Kb, Vb, off);
#pragma unroll 1
    for (int ch = 0; ch < nchunk; ++ch) {
        const bool last = ch == nchunk - 1;
        const int i_hi = last ? nfull : (ch + 1) * STEPS;          // a chunk before the last holds full row steps only
        float* sp = dense ? &stash[FILT ? 0 : ch & 1][(8 * w + r) * G] : nullptr;
#pragma unroll 1
        for (; i + 2 <= i_hi; i += 2, off += 2 * STEP) {
            load_tile(B, Kb, Vb, off + STEP);
            row_step<G>(st, qreg, A, sp, c, true);
            if (i + 2 < nfull) load_tile(A, Kb, Vb, off + 2 * STEP);
            row_step<G>(st, qreg, B, sp ? sp + 32 * G : nullptr, c, true);
            if (sp) sp += 64 * G;
        }
        if (last) {
            if (i < nfull) {
                row_step<G>(st, qreg, A, sp, c, true);
                if (sp) sp += 32 * G;
                ++i;
            }
            const int row = wave_row0 + 32 * i + r;                 // at most one ragged row step is left
            if (row - r < row_end) {
                const bool valid = row < row_end;
                load_tile(A, Kb, Vb, (uint32_t)(valid ? row : row_end - 1) * 256u + (uint32_t)c * 16u);
                row_step<G>(st, qreg, A, sp, c, valid);
            }
        }
        if (dense && FILT) {
            if (last) break;                 // the segment's last chunk is written out by the caller, behind the barrier it has anyway
            __syncthreads();
            seg_kept += write_kept<G>(stash[0], row_begin + ch * CAP, CAP, rep_base, kept_pos, row_begin + seg_kept, fc, sm_cnt,
                                      w, 8 * r + c);
            __syncthreads();                 // one staging buffer: the next chunk's rows wait until every wave has written this one's
        } else if (dense) {
            __syncthreads();
            const int first = row_begin + ch * CAP;
            const int nf = (row_end - first < CAP ? row_end - first : CAP) * G;     // floats of this chunk
            const float* src = stash[ch & 1];
            float* dst = rep_base + (size_t)first * G;                              // 128-byte aligned: first is a multiple of 32
            typedef float f4v __attribute__((ext_vector_type(4)));
            for (int f = (int)threadIdx.x * 4; f + 4 <= nf; f += 1024)      // streaming stores: nothing here reads them back
                __builtin_nontemporal_store(*reinterpret_cast<const f4v*>(src + f), reinterpret_cast<f4v*>(dst + f));
            for (int f = (nf & ~3) + (int)threadIdx.x; f < nf; f += 256) dst[f] = src[f];
        }
    }
    return seg_kept;
}

// What the filtered form of the split pass needs besides the arguments of the plain one.
struct FilterArgs {
    const RepFilter* filt;     // [n_reps] filter state, set by the monitor
    const RepDev* reps;        // [n_reps] for the candidate range of every pivot
    int32_t* surv_pos;         // [n_reps][max_ctx] positions of the kept rows, by segment
    int32_t* seg_cnt;          // [segments] kept rows of every pivot segment
    uint16_t* q_keep;          // [n_reps][G][D] copy of the pivots' queries (the monitor may have to score again)
};

template <int G, int WG_PER_CU, bool FILT>
__global__ __launch_bounds__(256, WG_PER_CU) void attn_split_kernel(const uint16_t* __restrict__ arena,
                                                                    const uint16_t* __restrict__ q,
                                                                    const BlkDev* __restrict__ blks,
                                                                    const SegDev* __restrict__ segs,
                                                                    float* __restrict__ part_acc,
                                                                    float* __restrict__ part_ml,
                                                                    float* __restrict__ rep_logits, int max_ctx,
                                                                    unsigned long long* __restrict__ stamps, FilterArgs fa)
{
    __shared__ float sm_m[4][G];
    __shared__ float sm_Z[16][G];
    __shared__ __attribute__((aligned(16))) float sm_red[4][G * HC_D];
    __shared__ __attribute__((aligned(16))) float sm_stash[FILT ? 1 : 2][REP_STASH_FLOATS];
    __shared__ int sm_kept[4];       // filtered: rows every wave keeps of the current chunk

    const int tid = threadIdx.x;
    const int w = tid >> 6;
    const int lane = tid & 63;
    const int r = lane >> 3;     // row inside a row step
    const int c = lane & 7;      // column lane

    // tuning runs only: when the workgroup started and (below) when it was through its last rows
    if (stamps && threadIdx.x == 0) stamps[2 * blockIdx.x] = __builtin_amdgcn_s_memrealtime();
    const BlkDev blk = blks[blockIdx.x];
    SegDev seg = blk.first;
    int next_extra = blk.extra_begin;
    for (;;) {
        const char* __restrict__ Kp = reinterpret_cast<const char*>(arena + seg.k_off);
        const char* __restrict__ Vp = reinterpret_cast<const char*>(arena + seg.v_off);
        float* rep_base = nullptr;
        int32_t* kept_pos = nullptr;
        int32_t* kept_count = nullptr;
        FilterCtx<G> fc;
        fc.cutsum = 0.f;
        fc.lo = fc.hi = 0;
#pragma unroll
        for (int g = 0; g < G; ++g) fc.ref[g] = 0.f;
        if (rep_logits && seg.rep_slot >= 0) {
            rep_base = rep_logits + (size_t)seg.rep_slot * G * max_ctx;
            if (FILT) {
                kept_pos = fa.surv_pos + (size_t)seg.rep_slot * max_ctx;
                kept_count = fa.seg_cnt + seg.slot;
                const RepFilter f = fa.filt[seg.rep_slot];
                fc.cutsum = f.cutsum;
#pragma unroll
                for (int g = 0; g < G; ++g) fc.ref[g] = f.ref[g];
                fc.lo = fa.reps[seg.rep_slot].lo;
                fc.hi = fa.reps[seg.rep_slot].hi;
                if (seg.row_begin == 0 && tid < G * 16)      // the pivot's queries, kept for the monitor: G rows of 16 x 16 bytes
                    reinterpret_cast<uint4*>(fa.q_keep + (size_t)seg.rep_slot * G * HC_D)[tid] =
                        reinterpret_cast<const uint4*>(q + (size_t)seg.bh * G * HC_D)[tid];
            }
        }

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

        int seg_kept = process_rows<G, FILT>(st, qreg, Kp, Vp, rep_base, fc, kept_pos, sm_stash, sm_kept, seg.row_begin, seg.row_end, w, r, c);
        if (stamps && threadIdx.x == 0 && next_extra >= blk.extra_end && st.Z[0] >= 0.f)      // (the condition on Z orders the stamp after the rows)
            stamps[2 * blockIdx.x + 1] = __builtin_amdgcn_s_memrealtime();

        // ---- merge the 4 waves x 8 row lanes into one partial ----
        // Inside a wave the 16 G accumulators of a lane are summed over the wave's 8 row lanes in registers:
        // lanes 8 apart by a DPP rotate, then rows of 16 lanes and halves of 32 lanes by the lane-swap
        // instructions, which reduce TWO registers at a time (afterwards the lanes with lane bit 4 clear
        // hold the sums of the first register, those with it set the sums of the second; bit 5 likewise), so
        // the 16 G registers shrink to 4 G and every lane is left with a quarter of the (head, column) sums:
        // flat index e + 4 G * [bit 5] + 8 G * [bit 4], e < 4 G, of acc[flat / 16][flat % 16].
        // The four waves' sums, each still relative to its own reference maximum, meet in LDS; one barrier.
        constexpr int NA = 16 * G;
        float red[NA / 4];
        {
            float half[NA / 2];
#pragma unroll
            for (int e = 0; e < NA / 2; ++e) {
                float x = st.acc[e / 16][e % 16], y = st.acc[(e + NA / 2) / 16][(e + NA / 2) % 16];
                x += dpp<DPP_ROR8>(x);
                y += dpp<DPP_ROR8>(y);
                swap_rows16(x, y);
                half[e] = x + y;
            }
#pragma unroll
            for (int e = 0; e < NA / 4; ++e) {
                float x = half[e], y = half[e + NA / 4];
                swap_halves32(x, y);
                red[e] = x + y;
            }
        }
        const int sel = ((lane >> 4) & 1) * 2 + (lane >> 5);          // [bit 4] * 2 + [bit 5]
        if ((lane & 8) == 0) {                                          // lanes 8 apart hold the same sums
            const int flat0 = (NA / 4) * sel;
#pragma unroll
            for (int e = 0; e < NA / 4; e += 4) {
                const int flat = flat0 + e, g = flat / 16, i = flat % 16;
                *reinterpret_cast<float4*>(&sm_red[w][g * HC_D + 64 * (i / 8) + 8 * c + (i % 8)]) =
                    make_float4(red[e], red[e + 1], red[e + 2], red[e + 3]);
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float z = st.Z[g];
            z += dpp<DPP_ROR8>(z);
            if ((lane & 15) == 0) sm_Z[w * 4 + sel][g] = z;            // one lane per row pair: c == 0, bit 3 clear
        }
        if (lane == 0) {
#pragma unroll
            for (int g = 0; g < G; ++g) sm_m[w][g] = st.m[g];
        }
        __syncthreads();
        for (int o = tid; o < G * HC_D; o += 256) {
            const int g = o / HC_D;
            const float M = fmaxf(fmaxf(sm_m[0][g], sm_m[1][g]), fmaxf(sm_m[2][g], sm_m[3][g]));
            float a = 0.f;
#pragma unroll
            for (int p = 0; p < 4; ++p) a += sm_red[p][o] * __builtin_amdgcn_exp2f(sm_m[p][g] - M);
            part_acc[(size_t)seg.slot * G * HC_D + o] = a;
        }
        if (tid < G) {
            const float M = fmaxf(fmaxf(sm_m[0][tid], sm_m[1][tid]), fmaxf(sm_m[2][tid], sm_m[3][tid]));
            float z = 0.f;
#pragma unroll
            for (int p = 0; p < 16; ++p) z += sm_Z[p][tid] * __builtin_amdgcn_exp2f(sm_m[p / 4][tid] - M);
            part_ml[((size_t)seg.slot * G + tid) * 2 + 0] = M;
            part_ml[((size_t)seg.slot * G + tid) * 2 + 1] = z;
        }
        if (FILT && rep_base) {          // the last chunk's kept rows (the barrier above followed its last staged row)
            constexpr int CAP = REP_STASH_FLOATS / G;
            const int lastc = (seg.row_end - seg.row_begin - 1) / CAP;
            const int first = seg.row_begin + lastc * CAP;
            seg_kept += write_kept<G>(sm_stash[0], first, seg.row_end - first, rep_base, kept_pos, seg.row_begin + seg_kept, fc,
                                      sm_kept, w, lane);
            if (tid == 0) *kept_count = seg_kept;
        }
        if (next_extra >= blk.extra_end) break;
        __syncthreads();
        seg = segs[next_extra++];
    }
}

// Second pass: out = sum_s 2^(m_s - M) acc_s / sum_s 2^(m_s - M) Z_s over the partials of one head.
// One workgroup per (b, query head, quarter of the columns): 32 partial lanes x CQ column quads; every thread's
// loads are independent and issued together.  (Four small workgroups per query head instead of one of 1024
// threads: they find room beside the monitor's kernels sooner.)
constexpr int CQ = 8;                       // column quads (of 32) per workgroup
constexpr int COMBINE_BLK = 32 * CQ;
template <int G>
__global__ __launch_bounds__(COMBINE_BLK) void attn_combine_kernel(const HeadDev* __restrict__ heads,
                                                                   const float* __restrict__ part_acc,
                                                                   const float* __restrict__ part_ml,
                                                                   float* __restrict__ out, float* __restrict__ lse)
{
    __shared__ float sm_max[COMBINE_BLK / 64];
    __shared__ float4 sm_acc[32][CQ];
    __shared__ float sm_z[32];
    const int bh = blockIdx.x / G, g = blockIdx.x % G;
    const HeadDev hd = heads[bh];
    const int tid = threadIdx.x, dq = (tid % CQ) + CQ * blockIdx.y, pl = tid / CQ;
    const int n = hd.part_count;
    const float2* ml = reinterpret_cast<const float2*>(part_ml);
    const float4* pa = reinterpret_cast<const float4*>(part_acc);

    // The first 128 partials' loads do not depend on the common maximum: they are issued before it is known,
    // so that the pass costs two memory round trips (descriptor, then everything) instead of three.
    float2 mz[4];
    float4 a[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int s = pl + 32 * u;
        const size_t slot = (size_t)(hd.part_begin + (s < n ? s : 0));
        mz[u] = ml[slot * G + g];
        a[u] = pa[(slot * G + g) * (HC_D / 4) + dq];
    }
    float mx = M_INIT;
    for (int s = tid; s < n; s += COMBINE_BLK) mx = fmaxf(mx, ml[(size_t)(hd.part_begin + s) * G + g].x);
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if ((tid & 63) == 0) sm_max[tid >> 6] = mx;
    __syncthreads();
    float M = sm_max[0];
#pragma unroll
    for (int i = 1; i < COMBINE_BLK / 64; ++i) M = fmaxf(M, sm_max[i]);

    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float z = 0.f;
    for (int s0 = pl; s0 < n; s0 += 128) {
        if (s0 != pl) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int s = s0 + 32 * u;
                const size_t slot = (size_t)(hd.part_begin + (s < n ? s : 0));
                mz[u] = ml[slot * G + g];
                a[u] = pa[(slot * G + g) * (HC_D / 4) + dq];
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float wgt = (s0 + 32 * u < n) ? __builtin_amdgcn_exp2f(mz[u].x - M) : 0.f;
            z += wgt * mz[u].y;
            acc.x += wgt * a[u].x;
            acc.y += wgt * a[u].y;
            acc.z += wgt * a[u].z;
            acc.w += wgt * a[u].w;
        }
    }
    sm_acc[pl][tid % CQ] = acc;
    if (tid % CQ == 0) sm_z[pl] = z;
    __syncthreads();
    if (tid < 4 * CQ) {     // column tid of this workgroup's 4 CQ: quad tid / 4, component tid % 4
        const float* col = reinterpret_cast<const float*>(&sm_acc[0][0]) + tid;
        float a = 0.f, zz = 0.f;
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            a += col[i * 4 * CQ];
            zz += sm_z[i];
        }
        out[(size_t)blockIdx.x * HC_D + 4 * CQ * blockIdx.y + tid] = a / zz;
        if (tid == 0 && blockIdx.y == 0) lse[blockIdx.x] = (M + __builtin_amdgcn_logf(zz)) * LN2;
    }
}

// Workgroups per compute unit the kernel is compiled for.  A wave keeps two tiles of 8 rows (4 KB each) in
// flight; the group-of-4 case holds 32 query + 64 accumulator registers, and two workgroups (8 waves)
// per compute unit keep 64 KB in flight there, which measurement shows is enough.
template <int G> struct Tune { static constexpr int WG = 2; };
template <> struct Tune<8> { static constexpr int WG = 1; };

// The pivots' logits over again, every row, into the dense [ctx][G] layout: what the monitor falls back on when
// its check of a filtered step fails (need[rep] != 0; evaluated on the device, so the launch is unconditional and
// normally finds nothing to do).  Same plan, same lanes, same dot products in the same order as the split pass,
// so the logits are bit for bit those an unfiltered pass would have stored.  Queries come from the copy the
// split pass kept.  Rare: plain stores, no staging.
struct RepLogitsItem {
    const uint16_t* arena;
    const uint16_t* q_keep;
    const BlkDev* blks;
    const SegDev* segs;
    float* rep_logits;
    const int32_t* need;
    int n_blocks, n_reps;
};
struct RepLogitsBatch {
    RepLogitsItem it[HC_MAX_GROUP];      // blockIdx.y picks the layer
};

template <int G>
__global__ __launch_bounds__(256) void rep_logits_kernel(RepLogitsBatch batch, int max_ctx)
{
    const RepLogitsItem& item = batch.it[blockIdx.y];
    bool any = false;                                      // (a few words, read by every workgroup: the usual case is "none")
    for (int i = 0; i < item.n_reps; ++i) any |= item.need[i] != 0;
    if (!any) return;
    const uint16_t* __restrict__ arena = item.arena;
    const uint16_t* __restrict__ q_keep = item.q_keep;
    const BlkDev* __restrict__ blks = item.blks;
    const SegDev* __restrict__ segs = item.segs;
    float* __restrict__ rep_logits = item.rep_logits;
    const int32_t* __restrict__ need = item.need;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r = lane >> 3, c = lane & 7;
    // few workgroups (the launch is there at every step and normally has nothing to do): each takes every
    // gridDim.x-th workgroup share of the split pass's plan
    for (int share = blockIdx.x; share < item.n_blocks; share += gridDim.x) {
    const BlkDev blk = blks[share];
    SegDev seg = blk.first;
    int next_extra = blk.extra_begin;
    for (;;) {
        if (seg.rep_slot >= 0 && need[seg.rep_slot] != 0) {
            const char* __restrict__ Kp = reinterpret_cast<const char*>(arena + seg.k_off);
            float* rep_base = rep_logits + (size_t)seg.rep_slot * G * max_ctx;
            uint32_t qreg[G][8];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const uint4* qp = reinterpret_cast<const uint4*>(q_keep + ((size_t)seg.rep_slot * G + g) * HC_D);
                const uint4 a = qp[c], b = qp[8 + c];
                qreg[g][0] = a.x; qreg[g][1] = a.y; qreg[g][2] = a.z; qreg[g][3] = a.w;
                qreg[g][4] = b.x; qreg[g][5] = b.y; qreg[g][6] = b.z; qreg[g][7] = b.w;
            }
            for (int row0 = seg.row_begin + 8 * w; row0 < seg.row_end; row0 += 32) {
                const int row = row0 + r;
                const bool valid = row < seg.row_end;
                const uint32_t off = (uint32_t)(valid ? row : seg.row_end - 1) * 256u + (uint32_t)c * 16u;
                Tile t;
                t.k0 = *reinterpret_cast<const uint4*>(Kp + off);
                t.k1 = *reinterpret_cast<const uint4*>(Kp + off + 128);
                t.v0 = t.v1 = make_uint4(0u, 0u, 0u, 0u);
                float sc[G];
                qk<G>(qreg, t, sc);
                stash_rep<G>(rep_base + (size_t)row * G, sc, c, valid);
            }
        }
        if (next_extra >= blk.extra_end) break;
        seg = segs[next_extra++];
    }
    }
}

template <int G>
hc_status launch(hc_ctx* ctx, const hc_layer* L, const void* arena, const void* q, float* out, float* lse,
                 float* rep_logits, hipStream_t st, float* part_acc, float* part_ml)
{
    // The optional timing events are attached to the kernel's own dispatch, so that their distance is the
    // kernel's execution time (what a profiler's kernel trace reports), not launch latency plus execution.
    hipEvent_t ev_begin = nullptr, ev_end = nullptr;
    if (ctx->timing_next < ctx->timing.size()) {
        ev_begin = ctx->timing[ctx->timing_next].first;
        ev_end = ctx->timing[ctx->timing_next].second;
        ++ctx->timing_next;
    }
    const bool filtered = rep_logits != nullptr && hc_layer_filtered(ctx, L);
    const FilterArgs fa{L->filt, L->reps, L->surv_pos, L->seg_cnt, L->q_keep};
#define HC_LAUNCH(KERNEL)                                                                                         \
    hipExtLaunchKernelGGL(KERNEL, dim3(L->n_blocks), dim3(256), 0, st, ev_begin, ev_end, 0,                      \
                          (const uint16_t*)arena, (const uint16_t*)q, (const BlkDev*)L->blks,                    \
                          (const SegDev*)L->segs, part_acc, part_ml, rep_logits, ctx->cfg.max_ctx,                 \
                          ctx->tune_stamps, fa)
    if (filtered)
        HC_LAUNCH((attn_split_kernel<G, Tune<G>::WG, true>));
    else
        HC_LAUNCH((attn_split_kernel<G, Tune<G>::WG, false>));
#undef HC_LAUNCH
    HC_HIP(ctx, hipGetLastError());
    attn_combine_kernel<G><<<dim3(L->n_heads * G, 32 / CQ), dim3(COMBINE_BLK), 0, st>>>(L->heads, part_acc, part_ml, out, lse);
    HC_HIP(ctx, hipGetLastError());
    return HC_OK;
}

template <int G>
hc_status launch_rep_logits(hc_ctx* ctx, int n, const hc_layer* const* layers, const void* const* arenas, float* const* rep_logits,
                            hipStream_t st)
{
    RepLogitsBatch batch{};
    int max_blocks = 0;
    for (int i = 0; i < n; ++i) {
        const hc_layer* L = layers[i];
        batch.it[i] = RepLogitsItem{(const uint16_t*)arenas[i], L->q_keep, L->blks, L->segs, rep_logits[i], L->need, L->n_blocks, L->n_reps};
        max_blocks = std::max(max_blocks, L->n_blocks);
    }
    rep_logits_kernel<G><<<dim3(std::min(max_blocks, 64), n), dim3(256), hc_side_lds(ctx, (const void*)rep_logits_kernel<G>, 0), st>>>(batch, ctx->cfg.max_ctx);
    HC_HIP(ctx, hipGetLastError());
    return HC_OK;
}

}   // namespace

// Fixed scratch for callers that cannot allocate: room for the split-K partial results of the largest plan
// hc_decode_attn_static accepts, HC_STATIC_MAX_PARTIALS slots of (accumulators [8][128], then (max, sum) [8][2]
// behind all accumulators).  One copy per GPU, held until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress: kernels get the address that call returns.
constexpr size_t STATIC_ACC_FLOATS = (size_t)HC_STATIC_MAX_PARTIALS * 8 * HC_D;
constexpr size_t STATIC_ML_FLOATS = (size_t)HC_STATIC_MAX_PARTIALS * 8 * 2;
static __device__ __align__(256) float scratch[STATIC_ACC_FLOATS + STATIC_ML_FLOATS];

hc_status hc_attn_static_scratch(hc_ctx* ctx, float** base)
{
    // once per context, with the context's device current (hc_create): every GPU holds its own copy of the array
    // at its own address
    void* ptr = nullptr;
    HC_HIP(ctx, hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    *base = static_cast<float*>(ptr);
    return HC_OK;
}

static hc_status launch_any(hc_ctx* ctx, const hc_layer* L, const void* arena, const void* q, float* out, float* lse,
                            float* rep_logits, hipStream_t st, float* part_acc, float* part_ml)
{
    switch (ctx->G) {
    case 1: return launch<1>(ctx, L, arena, q, out, lse, rep_logits, st, part_acc, part_ml);
    case 2: return launch<2>(ctx, L, arena, q, out, lse, rep_logits, st, part_acc, part_ml);
    case 4: return launch<4>(ctx, L, arena, q, out, lse, rep_logits, st, part_acc, part_ml);
    case 8: return launch<8>(ctx, L, arena, q, out, lse, rep_logits, st, part_acc, part_ml);
    }
    return hc_fail(ctx, HC_ESHAPE, "unsupported group size");
}

hc_status hc_launch_attn(hc_ctx* ctx, const hc_layer* L, const void* arena, const void* q, float* out, float* lse,
                         float* rep_logits, hipStream_t st)
{
    if ((size_t)L->n_partials > ctx->part_slots) return hc_fail(ctx, HC_ESTATE, "split-K workspace smaller than the plan");
    return launch_any(ctx, L, arena, q, out, lse, rep_logits, st, ctx->part_acc, ctx->part_ml);
}

hc_status hc_launch_attn_static(hc_ctx* ctx, const hc_layer* L, const void* arena, const void* q, float* out, float* lse,
                                float* rep_logits, hipStream_t st)
{
    if (!ctx->static_scratch) return hc_fail(ctx, HC_ESTATE, "hc_decode_attn_static: the fixed scratch array was not found on this device");
    if (L->n_partials > HC_STATIC_MAX_PARTIALS)
        return hc_fail(ctx, HC_ESHAPE, "hc_decode_attn_static: the layer's plan has %d partial results, the fixed scratch holds %d",
                       L->n_partials, (int)HC_STATIC_MAX_PARTIALS);
    return launch_any(ctx, L, arena, q, out, lse, rep_logits, st, ctx->static_scratch, ctx->static_scratch + STATIC_ACC_FLOATS);
}

hc_status hc_launch_rep_logits(hc_ctx* ctx, int n, const hc_layer* const* layers, const void* const* arenas, float* const* rep_logits,
                               hipStream_t st)
{
    if (n < 1 || n > HC_MAX_GROUP) return hc_fail(ctx, HC_EINVAL, "batch of %d layers", n);
    switch (ctx->G) {
    case 1: return launch_rep_logits<1>(ctx, n, layers, arenas, rep_logits, st);
    case 2: return launch_rep_logits<2>(ctx, n, layers, arenas, rep_logits, st);
    case 4: return launch_rep_logits<4>(ctx, n, layers, arenas, rep_logits, st);
    case 8: return launch_rep_logits<8>(ctx, n, layers, arenas, rep_logits, st);
    }
    return hc_fail(ctx, HC_ESHAPE, "unsupported group size");
}

hc_status hc_attn_set_lds_limit()
{
    const void* fns[] = {(const void*)rep_logits_kernel<1>, (const void*)rep_logits_kernel<2>, (const void*)rep_logits_kernel<4>,
                         (const void*)rep_logits_kernel<8>};
    for (const void* fn : fns)
        if (hc_allow_lds(fn) != hipSuccess) return HC_EHIP;
    return HC_OK;
}
