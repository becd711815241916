// hc_probe.hip -- two plain streaming kernels that measure what the machine at hand can give the hot path:
// the read bandwidth of HBM (the bound of the attention pass) and the read bandwidth of pinned host memory
// from a kernel (the bound of the gather, which reads the host tier over the host link the same way).
// They compute nothing of the method; bench.py times them beside the kernels they bound.
#include "hc_internal.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Every thread reads 16 bytes per step with a stride of the whole grid (coalesced, streaming loads) and folds
// them into one word, stored only if it takes a value it cannot take in practice: the loads stay, no store does.
template <bool NT>
__device__ __forceinline__ u32x4 ld16(const u32x4* p)
{
    return NT ? __builtin_nontemporal_load(p) : *p;
}

template <bool NT>
__global__ __launch_bounds__(256) void probe_stream_read(const u32x4* __restrict__ src, size_t n16, uint32_t* __restrict__ sink)
{
    uint32_t acc = 0;
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {          // four loads in flight per thread
        const u32x4 a = ld16<NT>(src + i), b = ld16<NT>(src + i + stride), c = ld16<NT>(src + i + 2 * stride),
                    d = ld16<NT>(src + i + 3 * stride);
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < n16; i += stride) {
        const u32x4 a = ld16<NT>(src + i);
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == 0x9e3779b9u && sink) sink[0] = acc;
}

// Pinned host memory -> HBM, 16 bytes per thread and step, eight loads in flight per thread before the first store.
__global__ __launch_bounds__(256) void probe_host_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 7 * stride < n16; i += 8 * stride) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 8; ++u) dst[i + u * stride] = v[u];
    }
    for (; i < n16; i += stride) dst[i] = __builtin_nontemporal_load(src + i);
}

}   // namespace

extern "C" hc_status hc_probe_stream_read(const void* dev_buf, size_t bytes, void* dev_sink, int32_t workgroups, int32_t streaming,
                                          void* stream)
{
    if (!dev_buf || ((uintptr_t)dev_buf & 15) || bytes < 16 || workgroups < 1 || workgroups > (1 << 20)) return HC_EINVAL;
    if (streaming)
        probe_stream_read<true><<<dim3(workgroups), dim3(256), 0, (hipStream_t)stream>>>((const u32x4*)dev_buf, bytes / 16, (uint32_t*)dev_sink);
    else
        probe_stream_read<false><<<dim3(workgroups), dim3(256), 0, (hipStream_t)stream>>>((const u32x4*)dev_buf, bytes / 16, (uint32_t*)dev_sink);
    return hipGetLastError() == hipSuccess ? HC_OK : HC_EHIP;
}

extern "C" hc_status hc_probe_host_copy(const void* pinned_src, void* dev_dst, size_t bytes, int32_t workgroups, void* stream)
{
    if (!pinned_src || !dev_dst || (((uintptr_t)pinned_src | (uintptr_t)dev_dst) & 15) || bytes < 16 || workgroups < 1 ||
        workgroups > (1 << 20))
        return HC_EINVAL;
    probe_host_copy<<<dim3(workgroups), dim3(256), 0, (hipStream_t)stream>>>((const u32x4*)pinned_src, (u32x4*)dev_dst, bytes / 16);
    return hipGetLastError() == hipSuccess ? HC_OK : HC_EHIP;
}
