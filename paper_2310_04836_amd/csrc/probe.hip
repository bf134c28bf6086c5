// Measurement aids, not part of the layer.
//
// (1) A plain streaming read of a device buffer with the
// same launch shape as the decode kernel (one 1024-thread workgroup per CU, 128-bit loads,
// several loads in flight per lane).  Its rate is the bandwidth a weight-streaming kernel
// could at best reach on this GPU for a buffer of that size.
//
// (2) A loop of nothing but v_mfma_i32_32x32x32_i8 on operands taken from a caller's buffer.
// The rate of the matrix cores depends on the operand DATA: the chip lowers its clock with the
// switching activity, so operands that look like real quantized tensors run well below the
// rate of constant operands.  This kernel measures the ceiling that applies to given data.
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

// Every lane takes four A and two B operands (96 bytes) from the buffer and then issues
// 8 * iters MFMAs on eight independent accumulators, no memory access in the loop.
__global__ __launch_bounds__(256) void mfma_rate_kernel(const uint4 *__restrict__ operands, size_t n_vec, int iters,
                                                        uint32_t *__restrict__ sink)
{
    const size_t gl = (size_t)blockIdx.x * 256 + threadIdx.x;
    v4i op[6];
#pragma unroll
    for (int i = 0; i < 6; ++i) {
        const uint4 v = operands[(gl * 6 + i) % n_vec];
        op[i] = v4i{(int)v.x, (int)v.y, (int)v.z, (int)v.w};
    }
    v16i acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(op[i >> 1], op[4 + (i & 1)], acc[i], 0, 0, 0);
    }
    uint32_t x = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) x ^= (uint32_t)acc[i][r] + 0x9E3779B9u * (uint32_t)(i * 16 + r + 1);
    if (x == 0x12345678u) sink[blockIdx.x] = x;  // keeps the sums alive; practically never true
}

}  // namespace

hipError_t launch_probe_mfma(const void *operands, size_t bytes, int iters, uint32_t *sink, int workgroups, hipStream_t st)
{
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(workgroups), dim3(256), 0, st, (const uint4 *)operands, bytes / 16, iters, sink);
    return hipGetLastError();
}

hipError_t launch_probe_read(const void *src, size_t bytes, uint32_t *sink, int workgroups, hipStream_t st)
{
    hipLaunchKernelGGL(stream_read_kernel, dim3(workgroups), dim3(1024), 0, st, (const uint4 *)src, bytes / 16, sink);
    return hipGetLastError();
}

}  // namespace dgq
