// A plain streaming copy, 16 bytes per lane: the measured roof beside which the conversion kernels are
// reported (they are HBM-bound codecs, so the rate of a copy with the same load and store width is what
// this GPU gives to a kernel that does nothing else).  Same launch shape as the row-wise kernels: a workgroup
// covers COPY_UNROLL runs of COPY_THREADS consecutive 16-byte chunks, every wave instruction contiguous.
#include "mxfp4_device.hpp"
#include "mxfp4_kernels.hpp"

namespace mxfp4 {

constexpr int COPY_THREADS = 256;
constexpr int COPY_UNROLL = 4;

template <bool NT_LOAD, bool NT_STORE>
__global__ void __launch_bounds__(COPY_THREADS) stream_copy_kernel(const u32x4 *src, u32x4 *dst, uint64_t n_chunks)
{
    const uint64_t c0 = (uint64_t)blockIdx.x * (COPY_THREADS * COPY_UNROLL) + threadIdx.x;
    u32x4 v[COPY_UNROLL];
#pragma unroll
    for (int u = 0; u < COPY_UNROLL; ++u) {
        const uint64_t c = c0 + (uint64_t)u * COPY_THREADS;
        if (c < n_chunks)
            v[u] = NT_LOAD ? __builtin_nontemporal_load(src + c) : src[c];
    }
#pragma unroll
    for (int u = 0; u < COPY_UNROLL; ++u) {
        const uint64_t c = c0 + (uint64_t)u * COPY_THREADS;
        if (c < n_chunks) {
            if (NT_STORE)
                __builtin_nontemporal_store(v[u], dst + c);
            else
                dst[c] = v[u];
        }
    }
}

hipError_t launch_stream_copy(const void *src, void *dst, int64_t bytes, int32_t policy, hipStream_t stream)
{
    const uint64_t n = (uint64_t)bytes / 16u;
    const dim3 grid((uint32_t)((n + COPY_THREADS * COPY_UNROLL - 1) / (COPY_THREADS * COPY_UNROLL)));
    const u32x4 *s = static_cast<const u32x4 *>(src);
    u32x4 *d = static_cast<u32x4 *>(dst);
    switch (policy) {
    case 0: hipLaunchKernelGGL((stream_copy_kernel<false, false>), grid, dim3(COPY_THREADS), 0, stream, s, d, n); break;
    case 1: hipLaunchKernelGGL((stream_copy_kernel<true, false>), grid, dim3(COPY_THREADS), 0, stream, s, d, n); break;
    case 2: hipLaunchKernelGGL((stream_copy_kernel<false, true>), grid, dim3(COPY_THREADS), 0, stream, s, d, n); break;
    default: hipLaunchKernelGGL((stream_copy_kernel<true, true>), grid, dim3(COPY_THREADS), 0, stream, s, d, n); break;
    }
    return hipGetLastError();
}

} // namespace mxfp4
