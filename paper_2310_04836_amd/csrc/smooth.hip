// Percentile clipping smoothing (Section 3.4, Eq. 6), offline and not on the timed path:
//     z_j = max_m |X[m][j]|,  t = the r-th largest z (r = ceil(pct * K), nearest rank),
//     k_j = max(z_j / t, 1);  then X' = X / k and W' = diag(k) W move the outliers' scale from
// the activations into the weights before these are quantized.
#include "dgq_device.hpp"

namespace dgq {
namespace {

__device__ __forceinline__ float ld_h(const uint16_t *p) { return (float)__builtin_bit_cast(_Float16, *p); }

// thread = one input channel, rows walked in sequence (coalesced across the block)
__global__ __launch_bounds__(256) void channel_absmax_kernel(const uint16_t *__restrict__ X, int M, int K,
                                                             float *__restrict__ z)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= K) return;
    float a = 0.0f;
    for (int m = 0; m < M; ++m) a = fmaxf(a, fabsf(ld_h(X + (size_t)m * K + j)));
    z[j] = a;
}

// One workgroup: radix select of the r-th largest z (non-negative floats order like their bit
// patterns), then k_j = max(z_j / t, 1) for every channel.
__global__ __launch_bounds__(1024) void smooth_select_kernel(const float *__restrict__ z, int K, int r,
                                                             float *__restrict__ k)
{
    __shared__ unsigned hist[256];
    __shared__ unsigned s_prefix, s_rank;
    unsigned prefix = 0;       // the bits of t found so far (from the top)
    unsigned rank = (unsigned)r;  // t is the rank-th largest among the values that match the prefix
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (threadIdx.x < 256) hist[threadIdx.x] = 0;
        __syncthreads();
        const unsigned himask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
        for (int j = threadIdx.x; j < K; j += 1024) {
            const unsigned b = __float_as_uint(z[j]);
            if ((b & himask) == (prefix & himask)) atomicAdd(&hist[(b >> shift) & 0xFFu], 1u);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            unsigned seen = 0;
            int d = 255;
            for (; d > 0; --d) {
                if (seen + hist[d] >= rank) break;
                seen += hist[d];
            }
            s_prefix = prefix | ((unsigned)d << shift);
            s_rank = rank - seen;
        }
        __syncthreads();
        prefix = s_prefix;
        rank = s_rank;
        __syncthreads();
    }
    const float t = __uint_as_float(prefix);
    for (int j = threadIdx.x; j < K; j += 1024) {
        const float q = t > 0.0f ? z[j] / t : 1.0f;
        k[j] = q < 1.0f ? 1.0f : q;
    }
}

__global__ __launch_bounds__(256) void smooth_weights_kernel(const uint16_t *__restrict__ W, const float *__restrict__ k,
                                                             int K, int N, uint16_t *__restrict__ Wout)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    for (int j = blockIdx.y; j < K; j += gridDim.y) {   // (a grid has at most 65535 rows of blocks)
        const size_t i = (size_t)j * N + n;
        float p = k[j] * ld_h(W + i);
        // keep the product and the rounding to fp16 two operations: fused into one mixed-precision
        // multiply-add with a +0 addend, a product of -0 would come out as +0
        asm volatile("" : "+v"(p));
        Wout[i] = __builtin_bit_cast(unsigned short, (_Float16)p);
    }
}

__global__ __launch_bounds__(256) void smooth_acts_kernel(const uint16_t *__restrict__ X, const float *__restrict__ k,
                                                          int M, int K, uint16_t *__restrict__ Xout)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= K) return;
    const float kj = k[j];
    for (int m = blockIdx.y; m < M; m += gridDim.y) {
        const size_t i = (size_t)m * K + j;
        Xout[i] = __builtin_bit_cast(unsigned short, (_Float16)(ld_h(X + i) / kj));
    }
}

}  // namespace

hipError_t launch_smooth_scales(const uint16_t *X, int M, int K, int r, float *k, float *z, hipStream_t st)
{
    hipLaunchKernelGGL(channel_absmax_kernel, dim3((K + 255) / 256), dim3(256), 0, st, X, M, K, z);
    hipLaunchKernelGGL(smooth_select_kernel, dim3(1), dim3(1024), 0, st, z, K, r, k);
    return hipGetLastError();
}

hipError_t launch_smooth_apply(const uint16_t *W, const uint16_t *X, const float *k, int M, int K, int N,
                               uint16_t *Wout, uint16_t *Xout, hipStream_t st)
{
    if (W) hipLaunchKernelGGL(smooth_weights_kernel, dim3((N + 255) / 256, K < 65535 ? K : 65535), dim3(256), 0, st, W, k, K, N, Wout);
    if (X) hipLaunchKernelGGL(smooth_acts_kernel, dim3((K + 255) / 256, M < 65535 ? M : 65535), dim3(256), 0, st, X, k, M, K, Xout);
    return hipGetLastError();
}

}  // namespace dgq
