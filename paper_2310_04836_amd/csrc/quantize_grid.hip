// Two-phase grid search of Section 3.3 (offline, not on the timed path), with the weight-only
// objective ||W - Q(W)||^2: there is no calibration set, so the activations of Eq. 3 and of
// the phase-2 objective are taken as the identity.  alpha runs over 1, 1 - step, ...,
// 1 - (n_alpha - 1) * step.
//
// Phase 1 (Eq. 3 with the 4-bit asymmetric quantizer of Eq. 1), one thread per (group, column):
//     lo = min(min W, 0), hi = max(max W, 0);  s = alpha * (hi - lo) / 15;
//     ZP = clamp(round(-(alpha * lo) / s), 0, 15);  u = clamp(round(W / s) + ZP, 0, 15);
//     the alpha with the smallest sum of (W - (u - ZP) * s)^2, the first on ties, gives S' and ZP.
// Phase 2 (Eq. 5 with the clip of Eq. 4): for every column the alpha that minimises the error of
// the whole column with s1 = alpha * max_j S'_j / 15, S2 = clamp(round(S' / s1), 1, 127),
// S = s1 * S2 and nibbles clipped to ZP +- floor(127 / S2); one thread per (column, alpha) sums
// the error in increasing k, a reduction over alpha picks the first minimum.  A last kernel
// writes S2 and the nibbles for the chosen s1.
//
// Every sum runs in increasing k in one thread and every '/' is one IEEE division (the library
// is built without fast-math and without contraction), so the integers are reproducible bit
// for bit by a plain CPU loop that follows the same text.
#include "dgq_device.hpp"

namespace dgq {
namespace {

__device__ __forceinline__ float ld_half(const uint16_t *p) { return (float)__builtin_bit_cast(_Float16, *p); }
__device__ __forceinline__ float clampf(float v, float lo, float hi) { return v < lo ? lo : (v > hi ? hi : v); }

__global__ __launch_bounds__(256) void grid_phase1_kernel(const uint16_t *__restrict__ W, int K, int N, int group,
                                                          int n_alpha, float step, float *__restrict__ sprime,
                                                          uint8_t *__restrict__ zp)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int j = blockIdx.y;
    if (n >= N) return;
    const uint16_t *col = W + (size_t)j * group * N + n;
    float lo = 0.0f, hi = 0.0f;
    for (int k = 0; k < group; ++k) {
        const float w = ld_half(col + (size_t)k * N);
        if (w < lo) lo = w;
        if (w > hi) hi = w;
    }
    float best_err = 0.0f, best_s = 0.0f;
    int best_zp = 0;
    bool have = false;
    if (hi - lo > 0.0f) {
        for (int i = 0; i < n_alpha; ++i) {
            const float alpha = 1.0f - (float)i * step;
            const float s = (alpha * (hi - lo)) / 15.0f;
            const float z = clampf(rintf(-(alpha * lo) / s), 0.0f, 15.0f);
            float err = 0.0f;
            for (int k = 0; k < group; ++k) {
                const float w = ld_half(col + (size_t)k * N);
                const float u = clampf(rintf(w / s) + z, 0.0f, 15.0f);
                const float d = w - (u - z) * s;
                err = err + d * d;
            }
            if (!have || err < best_err) {
                have = true;
                best_err = err;
                best_s = s;
                best_zp = (int)z;
            }
        }
    }
    sprime[(size_t)j * N + n] = best_s;
    zp[(size_t)j * N + n] = (uint8_t)best_zp;
}

// s1 candidate i of a column, and the error of the whole column under it
__device__ __forceinline__ float column_error(const uint16_t *__restrict__ W, const float *__restrict__ sprime,
                                              const uint8_t *__restrict__ zp, int K, int N, int group, int n,
                                              float c1)
{
    const int ng = K / group;
    float err = 0.0f;
    for (int j = 0; j < ng; ++j) {
        const float q2 = clampf(rintf(sprime[(size_t)j * N + n] / c1), 1.0f, 127.0f);
        const float S = c1 * q2;
        const int z = zp[(size_t)j * N + n];
        const int r = 127 / (int)q2;
        const float lo4 = (float)(z - r < 0 ? 0 : z - r), hi4 = (float)(z + r > 15 ? 15 : z + r);
        const uint16_t *col = W + (size_t)j * group * N + n;
        for (int k = 0; k < group; ++k) {
            const float w = ld_half(col + (size_t)k * N);
            const float u = clampf(rintf(w / S) + (float)z, lo4, hi4);
            const float d = w - (u - (float)z) * S;
            err = err + d * d;
        }
    }
    return err;
}

constexpr int kCols = 32;    // columns per block
constexpr int kALanes = 8;   // threads that share the alphas of one column

__global__ __launch_bounds__(kCols *kALanes) void grid_phase2_search_kernel(
    const uint16_t *__restrict__ W, const float *__restrict__ sprime, const uint8_t *__restrict__ zp, int K, int N,
    int group, int n_alpha, float step, float *__restrict__ s1)
{
    __shared__ float s_err[kALanes][kCols];
    __shared__ int s_idx[kALanes][kCols];
    const int c = threadIdx.x % kCols;
    const int y = threadIdx.x / kCols;
    const int n = blockIdx.x * kCols + c;
    const int ng = K / group;
    float smax = 0.0f;
    if (n < N)
        for (int j = 0; j < ng; ++j) smax = fmaxf(smax, sprime[(size_t)j * N + n]);
    float best_err = 0.0f;
    int best_i = -1;
    if (n < N && smax > 0.0f) {
        for (int i = y; i < n_alpha; i += kALanes) {
            const float alpha = 1.0f - (float)i * step;
            const float c1 = (alpha * smax) / 15.0f;
            const float err = column_error(W, sprime, zp, K, N, group, n, c1);
            if (best_i < 0 || err < best_err) {   // i increases: the first minimum of this lane stays
                best_err = err;
                best_i = i;
            }
        }
    }
    s_err[y][c] = best_err;
    s_idx[y][c] = best_i;
    __syncthreads();
    if (y != 0 || n >= N) return;
    for (int l = 1; l < kALanes; ++l) {
        const int i = s_idx[l][c];
        if (i < 0) continue;
        const float e = s_err[l][c];
        if (best_i < 0 || e < best_err || (e == best_err && i < best_i)) {  // first minimum over all alphas
            best_err = e;
            best_i = i;
        }
    }
    if (best_i < 0) {
        s1[n] = 1.0f;  // all-zero column
        return;
    }
    const float alpha = 1.0f - (float)best_i * step;
    s1[n] = (alpha * smax) / 15.0f;
}

__global__ __launch_bounds__(256) void grid_phase2_apply_kernel(const uint16_t *__restrict__ W,
                                                                const float *__restrict__ sprime,
                                                                const uint8_t *__restrict__ zp,
                                                                const float *__restrict__ s1, int K, int N,
                                                                int group, uint8_t *__restrict__ s2,
                                                                uint8_t *__restrict__ u4)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int j = blockIdx.y;
    if (n >= N) return;
    const float c1 = s1[n];
    const float q2 = clampf(rintf(sprime[(size_t)j * N + n] / c1), 1.0f, 127.0f);
    const float S = c1 * q2;
    const int z = zp[(size_t)j * N + n];
    const int r = 127 / (int)q2;
    const float lo4 = (float)(z - r < 0 ? 0 : z - r), hi4 = (float)(z + r > 15 ? 15 : z + r);
    s2[(size_t)j * N + n] = (uint8_t)q2;
    const uint16_t *col = W + (size_t)j * group * N + n;
    uint8_t *dst = u4 + (size_t)j * group * N + n;
    for (int k = 0; k < group; ++k) {
        const float w = ld_half(col + (size_t)k * N);
        dst[(size_t)k * N] = (uint8_t)clampf(rintf(w / S) + (float)z, lo4, hi4);
    }
}


// ---- the same search with the activation-weighted objectives of Section 3.3 ---------------------
// Eq. 3 (phase 1, per group) and the objective printed with Eq. 5 (phase 2, per column) measure the
// error on the layer's output for calibration activations X [M][K] and their dequantized INT8 form
// X^ = sx * xq:   err = sum_m ( X[m,:] w  -  X^[m,:] Q(w) )^2   over the k of the group / the column.
// Each of the two products of a token is summed on its own in increasing k, the squares in
// increasing m, all fp32 without contraction: a plain CPU loop reproduces the integers bit for bit.
// A thread keeps the products of 32 tokens in registers while it walks k once (each candidate
// weight is dequantized once per 32 tokens), so the order of every sum stays the stated one.
constexpr int kTok = 32;

__global__ __launch_bounds__(256) void act_dequant_kernel(const int8_t *__restrict__ xq, const float *__restrict__ sx,
                                                          int M, int K, float *__restrict__ xh)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (size_t)M * K) return;
    xh[i] = sx[i / K] * (float)xq[i];
}

// xw1[j][m][n] = sum over group j of X[m][k] * W[k][n];  xw2[m][n] = the same over the whole column
__global__ __launch_bounds__(64) void act_products_kernel(const uint16_t *__restrict__ W, const uint16_t *__restrict__ X,
                                                          int M, int K, int N, int group, float *__restrict__ xw1,
                                                          float *__restrict__ xw2)
{
    const int n = blockIdx.x * 64 + threadIdx.x;
    const int m = blockIdx.y;
    if (n >= N) return;
    const int ng = K / group;
    float tc = 0.0f;
    for (int j = 0; j < ng; ++j) {
        float tg = 0.0f;
        for (int k = j * group; k < (j + 1) * group; ++k) {
            const float p = ld_half(X + (size_t)m * K + k) * ld_half(W + (size_t)k * N + n);
            tg = tg + p;
            tc = tc + p;
        }
        xw1[((size_t)j * M + m) * N + n] = tg;
    }
    xw2[(size_t)m * N + n] = tc;
}

__global__ __launch_bounds__(64) void grid_act_phase1_kernel(const uint16_t *__restrict__ W, const float *__restrict__ xh,
                                                             const float *__restrict__ xw1, int M, int K, int N,
                                                             int group, int n_alpha, float step,
                                                             float *__restrict__ sprime, uint8_t *__restrict__ zp)
{
    const int n = blockIdx.x * 64 + threadIdx.x;
    const int j = blockIdx.y;
    if (n >= N) return;
    const uint16_t *col = W + (size_t)j * group * N + n;
    float lo = 0.0f, hi = 0.0f;
    for (int k = 0; k < group; ++k) {
        const float w = ld_half(col + (size_t)k * N);
        if (w < lo) lo = w;
        if (w > hi) hi = w;
    }
    float best_err = 0.0f, best_s = 0.0f;
    int best_zp = 0;
    bool have = false;
    if (hi - lo > 0.0f) {
        for (int i = 0; i < n_alpha; ++i) {
            const float alpha = 1.0f - (float)i * step;
            const float s = (alpha * (hi - lo)) / 15.0f;
            const float z = clampf(rintf(-(alpha * lo) / s), 0.0f, 15.0f);
            float err = 0.0f;
            for (int m0 = 0; m0 < M; m0 += kTok) {
                float t[kTok];
#pragma unroll
                for (int i2 = 0; i2 < kTok; ++i2) t[i2] = 0.0f;
                for (int k = 0; k < group; ++k) {
                    const float u = clampf(rintf(ld_half(col + (size_t)k * N) / s) + z, 0.0f, 15.0f);
                    const float wq = (u - z) * s;
                    const float *xr = xh + (size_t)m0 * K + (size_t)j * group + k;
#pragma unroll
                    for (int i2 = 0; i2 < kTok; ++i2)
                        if (m0 + i2 < M) t[i2] = t[i2] + xr[(size_t)i2 * K] * wq;
                }
#pragma unroll
                for (int i2 = 0; i2 < kTok; ++i2)
                    if (m0 + i2 < M) {
                        const float d = xw1[((size_t)j * M + m0 + i2) * N + n] - t[i2];
                        err = err + d * d;
                    }
            }
            if (!have || err < best_err) {
                have = true;
                best_err = err;
                best_s = s;
                best_zp = (int)z;
            }
        }
    }
    sprime[(size_t)j * N + n] = best_s;
    zp[(size_t)j * N + n] = (uint8_t)best_zp;
}

__device__ __forceinline__ float column_error_act(const uint16_t *__restrict__ W, const float *__restrict__ sprime,
                                                  const uint8_t *__restrict__ zp, const float *__restrict__ xh,
                                                  const float *__restrict__ xw2, int M, int K, int N, int group, int n,
                                                  float c1)
{
    const int ng = K / group;
    float err = 0.0f;
    for (int m0 = 0; m0 < M; m0 += kTok) {
        float t[kTok];
#pragma unroll
        for (int i2 = 0; i2 < kTok; ++i2) t[i2] = 0.0f;
        for (int j = 0; j < ng; ++j) {
            const float q2 = clampf(rintf(sprime[(size_t)j * N + n] / c1), 1.0f, 127.0f);
            const float S = c1 * q2;
            const int z = zp[(size_t)j * N + n];
            const int r = 127 / (int)q2;
            const float lo4 = (float)(z - r < 0 ? 0 : z - r), hi4 = (float)(z + r > 15 ? 15 : z + r);
            const uint16_t *col = W + (size_t)j * group * N + n;
            for (int k = 0; k < group; ++k) {
                const float u = clampf(rintf(ld_half(col + (size_t)k * N) / S) + (float)z, lo4, hi4);
                const float wq = (u - (float)z) * S;
                const float *xr = xh + (size_t)m0 * K + (size_t)j * group + k;
#pragma unroll
                for (int i2 = 0; i2 < kTok; ++i2)
                    if (m0 + i2 < M) t[i2] = t[i2] + xr[(size_t)i2 * K] * wq;
            }
        }
#pragma unroll
        for (int i2 = 0; i2 < kTok; ++i2)
            if (m0 + i2 < M) {
                const float d = xw2[(size_t)(m0 + i2) * N + n] - t[i2];
                err = err + d * d;
            }
    }
    return err;
}

__global__ __launch_bounds__(kCols *kALanes) void grid_act_phase2_search_kernel(
    const uint16_t *__restrict__ W, const float *__restrict__ sprime, const uint8_t *__restrict__ zp,
    const float *__restrict__ xh, const float *__restrict__ xw2, int M, int K, int N, int group, int n_alpha, float step,
    float *__restrict__ s1)
{
    __shared__ float s_err[kALanes][kCols];
    __shared__ int s_idx[kALanes][kCols];
    const int c = threadIdx.x % kCols;
    const int y = threadIdx.x / kCols;
    const int n = blockIdx.x * kCols + c;
    const int ng = K / group;
    float smax = 0.0f;
    if (n < N)
        for (int j = 0; j < ng; ++j) smax = fmaxf(smax, sprime[(size_t)j * N + n]);
    float best_err = 0.0f;
    int best_i = -1;
    if (n < N && smax > 0.0f) {
        for (int i = y; i < n_alpha; i += kALanes) {
            const float alpha = 1.0f - (float)i * step;
            const float c1 = (alpha * smax) / 15.0f;
            const float err = column_error_act(W, sprime, zp, xh, xw2, M, K, N, group, n, c1);
            if (best_i < 0 || err < best_err) {
                best_err = err;
                best_i = i;
            }
        }
    }
    s_err[y][c] = best_err;
    s_idx[y][c] = best_i;
    __syncthreads();
    if (y != 0 || n >= N) return;
    for (int l = 1; l < kALanes; ++l) {
        const int i = s_idx[l][c];
        if (i < 0) continue;
        const float e = s_err[l][c];
        if (best_i < 0 || e < best_err || (e == best_err && i < best_i)) {
            best_err = e;
            best_i = i;
        }
    }
    if (best_i < 0) {
        s1[n] = 1.0f;
        return;
    }
    const float alpha = 1.0f - (float)best_i * step;
    s1[n] = (alpha * smax) / 15.0f;
}

}  // namespace

hipError_t launch_quantize_grid(const uint16_t *W, int K, int N, int group, int n_alpha, float step, uint8_t *u4,
                                uint8_t *zp, uint8_t *s2, float *s1, float *sprime, hipStream_t st)
{
    const int ng = K / group;
    dim3 g1((N + 255) / 256, ng);
    hipLaunchKernelGGL(grid_phase1_kernel, g1, dim3(256), 0, st, W, K, N, group, n_alpha, step, sprime, zp);
    dim3 g2((N + kCols - 1) / kCols);
    hipLaunchKernelGGL(grid_phase2_search_kernel, g2, dim3(kCols * kALanes), 0, st, W, sprime, zp, K, N, group,
                       n_alpha, step, s1);
    hipLaunchKernelGGL(grid_phase2_apply_kernel, g1, dim3(256), 0, st, W, sprime, zp, s1, K, N, group, s2, u4);
    return hipGetLastError();
}

}  // namespace dgq

namespace dgq {

size_t quantize_grid_act_workspace_bytes(int M, int K, int N, int group)
{
    const size_t ng = (size_t)K / group;
    return sizeof(float) * (ng * N + (size_t)M * K + ng * M * N + (size_t)M * N);
}

hipError_t launch_quantize_grid_act(const uint16_t *W, const uint16_t *X, const int8_t *xq, const float *sx, int M, int K,
                                    int N, int group, int n_alpha, float step, uint8_t *u4, uint8_t *zp, uint8_t *s2,
                                    float *s1, float *workspace, hipStream_t st)
{
    const int ng = K / group;
    float *sprime = workspace;
    float *xh = sprime + (size_t)ng * N;
    float *xw1 = xh + (size_t)M * K;
    float *xw2 = xw1 + (size_t)ng * M * N;
    hipLaunchKernelGGL(act_dequant_kernel, dim3((unsigned)(((size_t)M * K + 255) / 256)), dim3(256), 0, st, xq, sx, M, K, xh);
    hipLaunchKernelGGL(act_products_kernel, dim3((N + 63) / 64, M), dim3(64), 0, st, W, X, M, K, N, group, xw1, xw2);
    hipLaunchKernelGGL(grid_act_phase1_kernel, dim3((N + 63) / 64, ng), dim3(64), 0, st, W, xh, xw1, M, K, N, group,
                       n_alpha, step, sprime, zp);
    hipLaunchKernelGGL(grid_act_phase2_search_kernel, dim3((N + kCols - 1) / kCols), dim3(kCols * kALanes), 0, st, W, sprime,
                       zp, xh, xw2, M, K, N, group, n_alpha, step, s1);
    hipLaunchKernelGGL(grid_phase2_apply_kernel, dim3((N + 255) / 256, ng), dim3(256), 0, st, W, sprime, zp, s1, K, N, group,
                       s2, u4);
    return hipGetLastError();
}

}  // namespace dgq
