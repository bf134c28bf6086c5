// Measurement aid, not part of the layer: a plain streaming read of a device buffer with the
// same launch shape as the decode kernel (one 1024-thread workgroup per CU, 128-bit loads,
// several loads in flight per lane).  Its rate is the bandwidth a weight-streaming kernel
// could at best reach on this GPU for a buffer of that size.
#include "dgq_device.hpp"

namespace dgq {
namespace {

constexpr int kDepth = 8;

__global__ __launch_bounds__(1024) void stream_read_kernel(const uint4 *__restrict__ src, size_t n_vec,
                                                           uint32_t *__restrict__ sink)
{
    // workgroup b reads the contiguous range [b, b+1) * n_vec / gridDim.x, 16 KiB per sweep
    const size_t per = (n_vec + gridDim.x - 1) / gridDim.x;
    const size_t lo = per * blockIdx.x;
    size_t hi = lo + per;
    if (hi > n_vec) hi = n_vec;
    uint32_t x = 0;
    size_t i = lo + threadIdx.x;
    for (; i + (size_t)(kDepth - 1) * 1024 < hi; i += (size_t)kDepth * 1024) {
        uint4 v[kDepth];
#pragma unroll
        for (int d = 0; d < kDepth; ++d) v[d] = src[i + (size_t)d * 1024];
#pragma unroll
        for (int d = 0; d < kDepth; ++d) x ^= v[d].x ^ v[d].y ^ v[d].z ^ v[d].w;
    }
    for (; i < hi; i += 1024) {
        const uint4 v = src[i];
        x ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    // keep the loads alive without a store per thread in the common case
    if (x == 0x9E3779B9u) sink[blockIdx.x] = x;
}

}  // namespace

hipError_t launch_probe_read(const void *src, size_t bytes, uint32_t *sink, int workgroups, hipStream_t st)
{
    hipLaunchKernelGGL(stream_read_kernel, dim3(workgroups), dim3(1024), 0, st, (const uint4 *)src, bytes / 16, sink);
    return hipGetLastError();
}

}  // namespace dgq
