// Per-token dynamic symmetric INT8 activation quantizer (Section 3.1 symmetric case with
// 8 bits; "per-token dynamic activation quantization", Section 4.1).
//
// One 256-thread workgroup per token.  The row is read once as 128-bit vectors of eight
// fp16 values and kept in registers; the absolute maximum is taken on the raw bit patterns
// (for non-negative fp16 numbers the integer order of the bits is the numeric order), reduced
// across the wavefront with data-parallel-primitive moves and across the four wavefronts through
// LDS; then every value is scaled, rounded to nearest-even and stored as eight packed bytes.
#include "dgq_device.hpp"

namespace dgq {
namespace {

constexpr int kThreads = 256;

// VPT > 0: each thread caches VPT vectors (K <= 2048 * VPT).  VPT == 0: any K, the row is read
// twice (the second read hits in cache).
template <int VPT>
__global__ __launch_bounds__(kThreads) void quant_act_kernel(const uint16_t *__restrict__ x, int M, int K,
                                                             int8_t *__restrict__ xq,
                                                             float *__restrict__ sx)
{
    __shared__ uint32_t wave_m[kThreads / 64];
    const int m = blockIdx.x;
    const int nvec = K >> 3;
    const uint4 *row = reinterpret_cast<const uint4 *>(x + (size_t)m * K);
    uint2 *dst = reinterpret_cast<uint2 *>(xq + (size_t)m * K);

    uint4 cache[VPT > 0 ? VPT : 1];
    uint32_t mx = 0;
    if (VPT > 0) {
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            int idx = threadIdx.x + i * kThreads;
            cache[i] = idx < nvec ? row[idx] : make_uint4(0, 0, 0, 0);
            mx = absmax_bits(cache[i], mx);
        }
    } else {
        for (int idx = threadIdx.x; idx < nvec; idx += kThreads) mx = absmax_bits(row[idx], mx);
    }
    mx = wave_max_u32_lane63(mx);
    if ((threadIdx.x & 63) == 63) wave_m[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = wave_m[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) mx = wave_m[w] > mx ? wave_m[w] : mx;

    const float a = half_bits_to_float(mx);
    float inv = 0.0f, s = 0.0f;
    if (a != 0.0f) {
        s = a / 127.0f;
        inv = 127.0f / a;
    }
    if (threadIdx.x == 0) sx[m] = s;
    // a == 0: inv = 0 makes every product +-0, which rounds to 0.
    if (VPT > 0) {
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            int idx = threadIdx.x + i * kThreads;
            if (idx < nvec) dst[idx] = quant_vec(cache[i], inv);
        }
    } else {
        for (int idx = threadIdx.x; idx < nvec; idx += kThreads) dst[idx] = quant_vec(row[idx], inv);
    }
}

// Gated-MLP producer fused with the per-token quantizer: h = fp16(float(silu(g) * u)) with silu and
// the product in fp64 (one rounding to fp32, one to fp16: the tensor a model would store between
// the two linear layers), then the same absmax / scale / round as quant_act_kernel on h.  GU is
// [M][2*I], gate columns first.  h never goes to memory.  Each thread keeps its VPT vectors of h
// (fp16 bits) in registers, so I <= 2048 * VPT.
__device__ __forceinline__ uint32_t silu_mul_pair(uint32_t g2, uint32_t u2)
{
    uint32_t r = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const double g = (double)half_bits_to_float((g2 >> (16 * h)) & 0xFFFFu);
        const double u = (double)half_bits_to_float((u2 >> (16 * h)) & 0xFFFFu);
        const double p = (g / (1.0 + exp(-g))) * u;
        const float p32 = (float)p;
        r |= (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)p32) << (16 * h);
    }
    return r;
}

template <int VPT>
__global__ __launch_bounds__(kThreads) void silu_mul_quant_act_kernel(const uint16_t *__restrict__ GU, int M, int I,
                                                                      int8_t *__restrict__ xq,
                                                                      float *__restrict__ sx)
{
    __shared__ uint32_t wave_m[kThreads / 64];
    const int m = blockIdx.x;
    const int nvec = I >> 3;
    const uint4 *grow = reinterpret_cast<const uint4 *>(GU + (size_t)m * 2 * I);
    const uint4 *urow = reinterpret_cast<const uint4 *>(GU + (size_t)m * 2 * I + I);
    uint2 *dst = reinterpret_cast<uint2 *>(xq + (size_t)m * I);

    uint4 cache[VPT];
    uint32_t mx = 0;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int idx = threadIdx.x + i * kThreads;
        cache[i] = make_uint4(0, 0, 0, 0);
        if (idx < nvec) {
            const uint4 g = grow[idx], u = urow[idx];
            cache[i] = make_uint4(silu_mul_pair(g.x, u.x), silu_mul_pair(g.y, u.y), silu_mul_pair(g.z, u.z),
                                  silu_mul_pair(g.w, u.w));
        }
        mx = absmax_bits(cache[i], mx);
    }
    mx = wave_max_u32_lane63(mx);
    if ((threadIdx.x & 63) == 63) wave_m[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = wave_m[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) mx = wave_m[w] > mx ? wave_m[w] : mx;
    const float a = half_bits_to_float(mx);
    float inv = 0.0f, s = 0.0f;
    if (a != 0.0f) {
        s = a / 127.0f;
        inv = 127.0f / a;
    }
    if (threadIdx.x == 0) sx[m] = s;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int idx = threadIdx.x + i * kThreads;
        if (idx < nvec) dst[idx] = quant_vec(cache[i], inv);
    }
}

// RMSNorm fused with the per-token quantizer: y = fp16(float(x * r * gamma)), r = 1/sqrt(mean x^2 + eps),
// everything up to the two roundings in fp64.  The sum of squares is added in fp64 in the fixed order
// described at sum_squares_f64 (shared with the decode kernel that normalises its own activations, so
// both give the same bits); that order differs from a running sum only in the last bits of a double,
// far below what survives the rounding to fp32 and fp16.  y is kept in registers as fp16 bits
// (K <= 2048 * VPT).
template <int VPT>
__global__ __launch_bounds__(kThreads) void rmsnorm_quant_act_kernel(const uint16_t *__restrict__ x,
                                                                     const uint16_t *__restrict__ gamma, int M, int K,
                                                                     float eps, int8_t *__restrict__ xq,
                                                                     float *__restrict__ sx)
{
    __shared__ double wave_s[kThreads / 64];
    __shared__ uint32_t wave_m[kThreads / 64];
    const int m = blockIdx.x;
    const int nvec = K >> 3;
    const uint4 *row = reinterpret_cast<const uint4 *>(x + (size_t)m * K);
    const uint4 *grow = reinterpret_cast<const uint4 *>(gamma);
    uint2 *dst = reinterpret_cast<uint2 *>(xq + (size_t)m * K);

    uint4 cache[VPT];
    double ss = 0.0;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int idx = threadIdx.x + i * kThreads;
        cache[i] = idx < nvec ? row[idx] : make_uint4(0, 0, 0, 0);
        ss += sum_squares_f64(cache[i]);     // the fixed order described at sum_squares_f64
    }
    ss = wave_sum_f64_lane63(ss);
    if ((threadIdx.x & 63) == 63) wave_s[threadIdx.x >> 6] = ss;
    __syncthreads();
    ss = wave_s[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) ss += wave_s[w];
    const double r = 1.0 / sqrt(ss / (double)K + (double)eps);

    uint32_t mx = 0;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int idx = threadIdx.x + i * kThreads;
        if (idx < nvec) {
            const uint4 g = grow[idx];
            const uint32_t w[4] = {cache[i].x, cache[i].y, cache[i].z, cache[i].w};
            const uint32_t gw[4] = {g.x, g.y, g.z, g.w};
            uint32_t y[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                y[k] = 0;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const double xv = (double)half_bits_to_float((w[k] >> (16 * h)) & 0xFFFFu);
                    const double gv = (double)half_bits_to_float((gw[k] >> (16 * h)) & 0xFFFFu);
                    const float p32 = (float)(xv * r * gv);
                    y[k] |= (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)p32) << (16 * h);
                }
            }
            cache[i] = make_uint4(y[0], y[1], y[2], y[3]);
        }
        mx = absmax_bits(cache[i], mx);
    }
    mx = wave_max_u32_lane63(mx);
    if ((threadIdx.x & 63) == 63) wave_m[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = wave_m[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) mx = wave_m[w] > mx ? wave_m[w] : mx;
    const float a = half_bits_to_float(mx);
    float inv = 0.0f, s = 0.0f;
    if (a != 0.0f) {
        s = a / 127.0f;
        inv = 127.0f / a;
    }
    if (threadIdx.x == 0) sx[m] = s;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int idx = threadIdx.x + i * kThreads;
        if (idx < nvec) dst[idx] = quant_vec(cache[i], inv);
    }
}

// Static tensor-wise scale (the "S" scheme of Section 4.1 / Table 5; symmetric form of Eq. 1 with
// 8 bits): xq = clamp(round(x / s), -127, 127) with one IEEE division per element, and every
// token's scale is s.  One thread per eight values; no reduction.
__global__ __launch_bounds__(kThreads) void quant_act_static_kernel(const uint16_t *__restrict__ x, size_t nvec,
                                                                    int M, float s, int8_t *__restrict__ xq,
                                                                    float *__restrict__ sx)
{
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < (size_t)M) sx[i] = s;
    if (i >= nvec) return;
    const uint4 v = reinterpret_cast<const uint4 *>(x)[i];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t b[8];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            float q = rintf(half_bits_to_float((w[k] >> (16 * h)) & 0xFFFFu) / s);
            q = fminf(fmaxf(q, -127.0f), 127.0f);
            b[2 * k + h] = (uint32_t)((int)q) & 0xFFu;
        }
    }
    uint2 r;
    r.x = b[0] | (b[1] << 8) | (b[2] << 16) | (b[3] << 24);
    r.y = b[4] | (b[5] << 8) | (b[6] << 16) | (b[7] << 24);
    reinterpret_cast<uint2 *>(xq)[i] = r;
}

}  // namespace

hipError_t launch_quant_act_static(const uint16_t *x, int M, int K, float s, int8_t *xq, float *sx, hipStream_t st)
{
    const size_t nvec = (size_t)M * (size_t)K / 8;   // K is a multiple of 128, so M <= nvec
    const size_t blocks = (nvec + kThreads - 1) / kThreads;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(quant_act_static_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, x, nvec, M, s, xq, sx);
    return hipGetLastError();
}

hipError_t launch_rmsnorm_quant_act(const uint16_t *x, const uint16_t *gamma, int M, int K, float eps, int8_t *xq,
                                    float *sx, hipStream_t st)
{
    dim3 grid(M), block(kThreads);
    const int nvec = K / 8;
    if (nvec <= 2 * kThreads)
        hipLaunchKernelGGL(rmsnorm_quant_act_kernel<2>, grid, block, 0, st, x, gamma, M, K, eps, xq, sx);
    else if (nvec <= 6 * kThreads)
        hipLaunchKernelGGL(rmsnorm_quant_act_kernel<6>, grid, block, 0, st, x, gamma, M, K, eps, xq, sx);
    else if (nvec <= 12 * kThreads)
        hipLaunchKernelGGL(rmsnorm_quant_act_kernel<12>, grid, block, 0, st, x, gamma, M, K, eps, xq, sx);
    else
        return hipErrorInvalidValue;   // K > 24576: checked by the caller
    return hipGetLastError();
}

hipError_t launch_silu_mul_quant_act(const uint16_t *GU, int M, int I, int8_t *xq, float *sx, hipStream_t st)
{
    dim3 grid(M), block(kThreads);
    const int nvec = I / 8;
    if (nvec <= 2 * kThreads)
        hipLaunchKernelGGL(silu_mul_quant_act_kernel<2>, grid, block, 0, st, GU, M, I, xq, sx);
    else if (nvec <= 6 * kThreads)
        hipLaunchKernelGGL(silu_mul_quant_act_kernel<6>, grid, block, 0, st, GU, M, I, xq, sx);
    else if (nvec <= 12 * kThreads)
        hipLaunchKernelGGL(silu_mul_quant_act_kernel<12>, grid, block, 0, st, GU, M, I, xq, sx);
    else
        return hipErrorInvalidValue;   // I > 24576: checked by the caller
    return hipGetLastError();
}

hipError_t launch_quant_act(const uint16_t *x, int M, int K, int8_t *xq, float *sx, hipStream_t st)
{
    dim3 grid(M), block(kThreads);
    const int nvec = K / 8;
    if (nvec <= 2 * kThreads)
        hipLaunchKernelGGL(quant_act_kernel<2>, grid, block, 0, st, x, M, K, xq, sx);
    else if (nvec <= 4 * kThreads)
        hipLaunchKernelGGL(quant_act_kernel<4>, grid, block, 0, st, x, M, K, xq, sx);
    else if (nvec <= 8 * kThreads)
        hipLaunchKernelGGL(quant_act_kernel<8>, grid, block, 0, st, x, M, K, xq, sx);
    else if (nvec <= 12 * kThreads)
        hipLaunchKernelGGL(quant_act_kernel<12>, grid, block, 0, st, x, M, K, xq, sx);
    else
        hipLaunchKernelGGL(quant_act_kernel<0>, grid, block, 0, st, x, M, K, xq, sx);
    return hipGetLastError();
}

}  // namespace dgq
