// Offline weight-side kernels: the round-to-nearest dual-grained quantizer (Table 1 "RTN",
// Section 3.1 symmetric scale, Eq. 5 scale decoupling), the packer that writes the device
// format of the Eq. 2 operands, and the test hook that expands them back to W_s8.
// None of these is on the timed path; they are written for coalesced access, not tuned.
#include "dgq_device.hpp"

namespace dgq {
namespace {

// ------------------------------------------------------------------------------------
// RTN-DGQ quantizer.  Block = 64 columns x 4 k-lanes.  Pass 1: absolute maximum of each
// column (max_j S'_j = (max_k |W|)/7 because x -> x/7 is monotone), pass 2: per group
// absolute maximum -> s2, then the nibbles.
// ------------------------------------------------------------------------------------
constexpr int kQCols = 64;
constexpr int kQLanes = 4;

__device__ __forceinline__ float load_half(const uint16_t *p)
{
    return (float)__builtin_bit_cast(_Float16, *p);
}

__global__ __launch_bounds__(kQCols *kQLanes) void quantize_rtn_kernel(
    const uint16_t *__restrict__ W, int K, int N, int group, int8_t *__restrict__ w4,
    uint8_t *__restrict__ s2, float *__restrict__ s1)
{
    __shared__ float colmax[kQLanes][kQCols];
    const int c = threadIdx.x % kQCols;
    const int y = threadIdx.x / kQCols;
    const int n = blockIdx.x * kQCols + c;
    const bool live = n < N;
    const int ng = K / group;

    float a = 0.0f;
    if (live)
        for (int k = y; k < K; k += kQLanes) a = fmaxf(a, fabsf(load_half(W + (size_t)k * N + n)));
    colmax[y][c] = a;
    __syncthreads();
    a = colmax[0][c];
#pragma unroll
    for (int i = 1; i < kQLanes; ++i) a = fmaxf(a, colmax[i][c]);
    if (!live) return;

    const float spmax = a / 7.0f;
    if (spmax == 0.0f) {
        if (y == 0) s1[n] = 1.0f;
        for (int j = y; j < ng; j += kQLanes) s2[(size_t)j * N + n] = 1;
        for (int k = y; k < K; k += kQLanes) w4[(size_t)k * N + n] = 0;
        return;
    }
    const float c1 = spmax / 15.0f;
    if (y == 0) s1[n] = c1;
    for (int j = y; j < ng; j += kQLanes) {
        const uint16_t *col = W + (size_t)j * group * N + n;
        float ga = 0.0f;
        for (int k = 0; k < group; ++k) ga = fmaxf(ga, fabsf(load_half(col + (size_t)k * N)));
        const float sp = ga / 7.0f;
        float q = rintf(sp / c1);
        q = fminf(fmaxf(q, 1.0f), 15.0f);
        s2[(size_t)j * N + n] = (uint8_t)q;
        const float S = c1 * q;
        int8_t *dst = w4 + (size_t)j * group * N + n;
        for (int k = 0; k < group; ++k) {
            float w = rintf(load_half(col + (size_t)k * N) / S);
            w = fminf(fmaxf(w, -8.0f), 7.0f);
            dst[(size_t)k * N] = (int8_t)w;
        }
    }
}

// ------------------------------------------------------------------------------------
// Packer.  Thread = one 16-byte cell = 32 consecutive k of one column.  threadIdx.x walks
// the columns (coalesced reads of w4 rows; 16 lanes write 256 contiguous bytes), blockIdx.y
// walks the 32-k blocks.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pack_cells_kernel(const int8_t *__restrict__ w4, int K, int N,
                                                         uint4 *__restrict__ qweight,
                                                         int32_t *__restrict__ bad_count)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int kk = blockIdx.y;  // 32-k block
    if (n >= N) return;
    const int8_t *src = w4 + (size_t)kk * 32 * N + n;
    uint32_t word[4] = {0, 0, 0, 0};
    int bad = 0;
#pragma unroll
    for (int r = 0; r < 32; ++r) {
        int w = src[(size_t)r * N];
        if (w < -8 || w > 7) {
            ++bad;
            w = 0;
        }
        const uint32_t u = (uint32_t)(w + 8);
        const int byte = r & 15;              // byte k%16 of the cell
        const int shift = (byte & 3) * 8 + (r >> 4) * 4;
        word[byte >> 2] |= u << shift;
    }
    const int ksteps = K >> 7;
    const size_t cell = ((size_t)(n >> 4) * ksteps + (kk >> 2)) * 64 + (size_t)(kk & 3) * 16 + (n & 15);
    qweight[cell] = make_uint4(word[0], word[1], word[2], word[3]);
    if (bad && bad_count) atomicAdd(bad_count, bad);
}

// Thread = four consecutive groups of one column -> one 32-bit word of `scales`.
__global__ __launch_bounds__(256) void pack_scales_kernel(const uint8_t *__restrict__ s2, int ng, int N,
                                                          uint32_t *__restrict__ scales,
                                                          int32_t *__restrict__ bad_count)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int gq = blockIdx.y;
    if (n >= N) return;
    const int gqn = (ng + 3) >> 2;
    uint32_t word = 0;
    int bad = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int gi = gq * 4 + i;
        if (gi < ng) {
            uint32_t s = s2[(size_t)gi * N + n];
            if (s < 1 || s > 15) {
                ++bad;
                s = 1;
            }
            word |= s << (8 * i);
        }
    }
    scales[((size_t)(n >> 4) * gqn + gq) * 16 + (n & 15)] = word;
    if (bad && bad_count) atomicAdd(bad_count, bad);
}

// ------------------------------------------------------------------------------------
// Packer for the general operands of Eq. 2: unsigned nibbles, group scales in [1, 127] and
// per-group zero points.  Same cells; the scale array holds (S2, ZP) byte pairs.  A nibble
// whose product S2 * (u - ZP) leaves INT8 (the constraint that Eq. 4 enforces) is counted and
// packed as ZP, i.e. as a zero weight.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pack_cells_zp_kernel(const uint8_t *__restrict__ u4,
                                                            const uint8_t *__restrict__ s2,
                                                            const uint8_t *__restrict__ zp, int K, int N,
                                                            int group, uint4 *__restrict__ qweight,
                                                            int32_t *__restrict__ bad_count)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int kk = blockIdx.y;  // 32-k block
    if (n >= N) return;
    const int gi = (kk * 32) / group;
    int s = s2[(size_t)gi * N + n], z = zp[(size_t)gi * N + n];
    if (s < 1 || s > 127) s = 1;  // counted by pack_scales_zp_kernel
    if (z > 15) z = 0;
    const uint8_t *src = u4 + (size_t)kk * 32 * N + n;
    uint32_t word[4] = {0, 0, 0, 0};
    int bad = 0;
#pragma unroll
    for (int r = 0; r < 32; ++r) {
        int u = src[(size_t)r * N];
        const int v = s * (u - z);
        if (u > 15 || v < -128 || v > 127) {
            ++bad;
            u = z;
        }
        const int byte = r & 15;
        const int shift = (byte & 3) * 8 + (r >> 4) * 4;
        word[byte >> 2] |= (uint32_t)u << shift;
    }
    const int ksteps = K >> 7;
    const size_t cell = ((size_t)(n >> 4) * ksteps + (kk >> 2)) * 64 + (size_t)(kk & 3) * 16 + (n & 15);
    qweight[cell] = make_uint4(word[0], word[1], word[2], word[3]);
    if (bad && bad_count) atomicAdd(bad_count, bad);
}

// Thread = two consecutive groups of one column -> one 32-bit word of (S2, ZP) pairs.
__global__ __launch_bounds__(256) void pack_scales_zp_kernel(const uint8_t *__restrict__ s2,
                                                             const uint8_t *__restrict__ zp, int ng, int N,
                                                             uint32_t *__restrict__ scales,
                                                             int32_t *__restrict__ bad_count)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int gh = blockIdx.y;
    if (n >= N) return;
    const int ghn = (ng + 1) >> 1;
    uint32_t word = 0;
    int bad = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int gi = gh * 2 + i;
        if (gi < ng) {
            uint32_t s = s2[(size_t)gi * N + n], z = zp[(size_t)gi * N + n];
            if (s < 1 || s > 127) {
                ++bad;
                s = 1;
            }
            if (z > 15) {
                ++bad;
                z = 0;
            }
            word |= (s | (z << 8)) << (16 * i);
        }
    }
    scales[((size_t)(n >> 4) * ghn + gh) * 16 + (n & 15)] = word;
    if (bad && bad_count) atomicAdd(bad_count, bad);
}

// ------------------------------------------------------------------------------------
// Unpack test hook: thread = one cell, expanded with the same device function the GEMM
// kernels use, written to W_s8[K][N].
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void unpack_kernel(const uint4 *__restrict__ qweight,
                                                     const uint32_t *__restrict__ scales, int zp_form,
                                                     int K, int N, int group, int8_t *__restrict__ w_s8)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int kk = blockIdx.y;
    if (n >= N) return;
    const int ksteps = K >> 7;
    const int ng = K / group;
    const ScaleForm sf = scale_form(zp_form);
    const int fsh = sf.fsh;
    const int gqn = (ng + (1 << fsh) - 1) >> fsh;
    const size_t cell = ((size_t)(n >> 4) * ksteps + (kk >> 2)) * 64 + (size_t)(kk & 3) * 16 + (n & 15);
    const uint4 q = qweight[cell];
    const int gi = (kk * 32) / group;
    const uint32_t sw = scales[((size_t)(n >> 4) * gqn + (gi >> fsh)) * 16 + (n & 15)];
    const GroupScale gs = group_scale_at(sw, scale_entry_shift(gi, sf), sf);
    v4i first, second;
    expand_cell(q, gs, first, second);
    int8_t *dst = w_s8 + (size_t)kk * 32 * N + n;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        dst[(size_t)r * N] = (int8_t)((first[r >> 2] >> (8 * (r & 3))) & 0xFF);
        dst[(size_t)(16 + r) * N] = (int8_t)((second[r >> 2] >> (8 * (r & 3))) & 0xFF);
    }
}

}  // namespace

hipError_t launch_quantize_rtn(const uint16_t *W, int K, int N, int group, int8_t *w4, uint8_t *s2,
                               float *s1, hipStream_t st)
{
    dim3 grid((N + kQCols - 1) / kQCols), block(kQCols * kQLanes);
    hipLaunchKernelGGL(quantize_rtn_kernel, grid, block, 0, st, W, K, N, group, w4, s2, s1);
    return hipGetLastError();
}

hipError_t launch_pack(const int8_t *w4, const uint8_t *s2, int K, int N, int group, void *qweight,
                       void *scales, int32_t *bad_count, hipStream_t st)
{
    const int ng = K / group;
    dim3 block(256);
    dim3 grid_c((N + 255) / 256, K / 32);
    hipLaunchKernelGGL(pack_cells_kernel, grid_c, block, 0, st, w4, K, N, (uint4 *)qweight, bad_count);
    dim3 grid_s((N + 255) / 256, (ng + 3) / 4);
    hipLaunchKernelGGL(pack_scales_kernel, grid_s, block, 0, st, s2, ng, N, (uint32_t *)scales, bad_count);
    return hipGetLastError();
}

hipError_t launch_pack_zp(const uint8_t *u4, const uint8_t *s2, const uint8_t *zp, int K, int N, int group,
                          void *qweight, void *scales_zp, int32_t *bad_count, hipStream_t st)
{
    const int ng = K / group;
    dim3 block(256);
    dim3 grid_c((N + 255) / 256, K / 32);
    hipLaunchKernelGGL(pack_cells_zp_kernel, grid_c, block, 0, st, u4, s2, zp, K, N, group, (uint4 *)qweight,
                       bad_count);
    dim3 grid_s((N + 255) / 256, (ng + 1) / 2);
    hipLaunchKernelGGL(pack_scales_zp_kernel, grid_s, block, 0, st, s2, zp, ng, N, (uint32_t *)scales_zp,
                       bad_count);
    return hipGetLastError();
}

hipError_t launch_unpack(const void *qweight, const void *scales, int zp_form, int K, int N, int group,
                         int8_t *w_s8, hipStream_t st)
{
    dim3 block(256);
    dim3 grid((N + 255) / 256, K / 32);
    hipLaunchKernelGGL(unpack_kernel, grid, block, 0, st, (const uint4 *)qweight, (const uint32_t *)scales,
                       zp_form, K, N, group, w_s8);
    return hipGetLastError();
}

}  // namespace dgq
