// Batched INT8 x INT8 -> INT32 matrix product for attention (Section 4.1, "Implementation": the
// attention products run as INT8 batched matrix multiplications), with the scale epilogue of
// Eq. 2: out[b][m][n] = fp16((sa[b][m] * sb[b][n]) * sum_k A[b][m][k] * B[b][n][k]).
//
// Both operands have k contiguous (scores: A = Q, B = K; context: A = P, B = V transposed), so
// both go the way the activations go in the tiled linear kernel: 128-byte rows in LDS, 16-byte
// unit u of row r stored at unit u ^ ((r/2) % 8), which makes the 128-bit reads of sixteen
// consecutive rows (one read phase of a v_mfma_i32_32x32x32_i8 operand) conflict-free.
//
//   - Workgroup tile 128 x 128, four wavefronts as 2 x 2, each 64 x 64 = 2 x 2 MFMA tiles of
//     32 x 32 (64 accumulation registers); K in stages of 128.
//   - Global -> registers -> LDS, double buffered: the loads of stage s + 1 are issued before
//     the MFMAs of stage s and written to the other LDS buffer after them; one barrier a stage.
//   - At the shapes of attention the product is bound by memory (the score matrix written, the
//     probability matrix read), not by the matrix cores, so nothing more elaborate is needed.
//   - Ragged M, N: rows past the end repeat the last row and are never stored.  K is a multiple
//     of 16; units past the end of K are zeros.
//   - M <= 16 (decode: one query token per head) takes another kernel, dot products on the vector
//     units, described where it stands.
#include "dgq_device.hpp"

namespace dgq {
namespace {

constexpr int BM = 128, BN = 128, BK = 128;

__device__ __forceinline__ int swz(int row, int unit) { return row * BK + ((unit ^ ((row >> 1) & 7)) << 4); }

// DB: two LDS buffers (K > 128).  A product with a single stage of K (attention scores: K is the head size)
// needs one, which lets three workgroups share a CU and overlap each other's loads, MFMAs and stores.
template <bool ACC, bool DB>
__global__ __launch_bounds__(256, DB ? 2 : 3) void bmm_s8_kernel(const int8_t *__restrict__ A, const int8_t *__restrict__ B,
                                                        const float *__restrict__ sa, const float *__restrict__ sb,
                                                        uint16_t *__restrict__ out, int32_t *__restrict__ acc_out, int M,
                                                        int N, int K)
{
    __shared__ __attribute__((aligned(16))) int8_t lds[DB ? 2 : 1][2][BM * BK];   // [buffer][operand][row * 128 + unit]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int kb = lane >> 5, li = lane & 31;
    const int n0 = blockIdx.x * BN, m0 = blockIdx.y * BM;
    const size_t batch = blockIdx.z;
    const int8_t *Ab = A + batch * (size_t)M * K;
    const int8_t *Bb = B + batch * (size_t)N * K;

    // this thread's four 16-byte units of each operand tile: rows tid/8 + 32*j, unit tid%8
    const int unit = tid & 7;
    const int8_t *arow[4], *brow[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = (tid >> 3) + 32 * j;
        int m = m0 + r, n = n0 + r;
        m = m < M ? m : M - 1;
        n = n < N ? n : N - 1;
        arow[j] = Ab + (size_t)m * K + unit * 16;
        brow[j] = Bb + (size_t)n * K + unit * 16;
    }
    uint4 ra[4], rb[4];
    auto load_stage = [&](int s) {
        const int k = s * BK + unit * 16;
        const bool in = k < K;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            ra[j] = in ? *reinterpret_cast<const uint4 *>(arow[j] + (size_t)s * BK) : make_uint4(0, 0, 0, 0);
            rb[j] = in ? *reinterpret_cast<const uint4 *>(brow[j] + (size_t)s * BK) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = (tid >> 3) + 32 * j;
            *reinterpret_cast<uint4 *>(&lds[buf][0][swz(r, unit)]) = ra[j];
            *reinterpret_cast<uint4 *>(&lds[buf][1][swz(r, unit)]) = rb[j];
        }
    };

    v16i acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    const int stages = (K + BK - 1) / BK;
    load_stage(0);
    store_stage(0);
    __syncthreads();
    for (int s = 0; s < stages; ++s) {
        const int buf = DB ? (s & 1) : 0;   // (without DB there is one stage)
        if (DB && s + 1 < stages) load_stage(s + 1);
#pragma unroll
        for (int g = 0; g < 4; ++g) {       // 32 k per MFMA: lane (kb, i) holds k = 32*g + 16*kb .. + 15 of row i
            v4i a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[i] = *reinterpret_cast<const v4i *>(&lds[buf][0][swz(wm * 64 + i * 32 + li, 2 * g + kb)]);
                b[i] = *reinterpret_cast<const v4i *>(&lds[buf][1][swz(wn * 64 + i * 32 + li, 2 * g + kb)]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (DB && s + 1 < stages) store_stage(buf ^ 1);
        __syncthreads();
    }

    // acc[i][j][r] of lane l: row m0 + wm*64 + i*32 + 8*(r/4) + 4*(l/32) + r%4, column n0 + wn*64 + j*32 + l%32
    if (ACC) {
        int32_t *dst = acc_out + batch * (size_t)M * N;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int n = n0 + wn * 64 + j * 32 + li;
                if (n >= N) continue;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * kb + (r & 3);
                    if (m < M) dst[(size_t)m * N + n] = acc[i][j][r];
                }
            }
        return;
    }
    // fp16: scaled values are transposed through LDS (32 rows x 64 columns per wavefront at a time) so
    // that a lane stores 16 contiguous bytes where the row stride allows it
    uint16_t *dst = out + batch * (size_t)M * N;
    float *lds_sa = reinterpret_cast<float *>(&lds[0][0][0]);                                  // 128 floats
    unsigned short *lds_t = reinterpret_cast<unsigned short *>(&lds[0][0][0] + 1024 + wave * 4096);
    if (tid < BM) lds_sa[tid] = (m0 + tid < M) ? (sa ? sa[batch * M + m0 + tid] : 1.0f) : 0.0f;
    float sbn[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int n = n0 + wn * 64 + j * 32 + li;
        sbn[j] = n < N ? (sb ? sb[batch * N + n] : 1.0f) : 0.0f;
    }
    __syncthreads();
    const bool vec = (N & 7) == 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 8 * (r >> 2) + 4 * kb + (r & 3);
                const float sc = lds_sa[wm * 64 + i * 32 + row] * sbn[j];
                lds_t[row * 64 + j * 32 + li] = scaled_sum_to_half_bits(sc, acc[i][j][r]);
            }
        // (a wavefront only reads back what it wrote itself: no barrier needed, the LDS operations of a
        // wavefront complete in order)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int row = q * 8 + (lane >> 3);
            const int m = m0 + wm * 64 + i * 32 + row;
            const int n = n0 + wn * 64 + (lane & 7) * 8;
            if (m >= M || n >= N) continue;
            if (vec) {
                // streaming store: the output is written once and read by another kernel; kept out of
                // the way of the operands in L2 (scores of LLaMA-7B prefill: 78 -> 62 us)
                __builtin_nontemporal_store(*reinterpret_cast<const v4i *>(&lds_t[row * 64 + (lane & 7) * 8]),
                                            reinterpret_cast<v4i *>(&dst[(size_t)m * N + n]));
            } else {
                for (int e = 0; e < 8 && n + e < N; ++e) dst[(size_t)m * N + n + e] = lds_t[row * 64 + (lane & 7) * 8 + e];
            }
        }
    }
}

// Few rows of A (one query token per head at decode): the product is a handful of dot products per
// row of B and is bound by reading B once, so no matrix instruction is needed.  A group of LPR lanes
// (a power of two, at least K / 16 and at most 64) owns one row n of B: a lane takes 16-byte pieces
// l, l + LPR, ... of it and of every row of A (v_dot4_i32_i8), the group adds its lanes' sums with
// lane exchanges, and its first lane writes the MT results.  A 256-thread workgroup covers 256 / LPR
// rows of B of one batch.
template <int MT, bool ACC>
__global__ __launch_bounds__(256) void bmm_s8_rows_kernel(const int8_t *__restrict__ A, const int8_t *__restrict__ B,
                                                         const float *__restrict__ sa, const float *__restrict__ sb,
                                                         uint16_t *__restrict__ out, int32_t *__restrict__ acc_out, int M,
                                                         int N, int K, int lpr_log2)
{
    const int lpr = 1 << lpr_log2;
    const int l = threadIdx.x & (lpr - 1);
    const int n = blockIdx.x * (256 >> lpr_log2) + (threadIdx.x >> lpr_log2);
    const size_t batch = blockIdx.y;
    const int pieces = K >> 4;
    const int8_t *Ab = A + batch * (size_t)M * K;
    const int8_t *Bn = B + (batch * (size_t)N + (n < N ? n : N - 1)) * K;   // rows past the end repeat the last one
    int acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[m] = 0;
    for (int p = l; p < pieces; p += lpr) {
        const v4i b = *reinterpret_cast<const v4i *>(Bn + (size_t)p * 16);
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            if (m < M) {
                const v4i a = *reinterpret_cast<const v4i *>(Ab + (size_t)m * K + (size_t)p * 16);
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[m] = __builtin_amdgcn_sdot4(a[q], b[q], acc[m], false);
            }
        }
    }
#pragma unroll
    for (int m = 0; m < MT; ++m)
        for (int d = lpr >> 1; d > 0; d >>= 1) acc[m] += __shfl_xor(acc[m], d, 64);
    if (l != 0 || n >= N) return;
    const float sbn = ACC ? 0.0f : (sb ? sb[batch * N + n] : 1.0f);
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        if (m >= M) break;
        const size_t o = (batch * (size_t)M + m) * N + n;
        if (ACC)
            acc_out[o] = acc[m];
        else
            out[o] = scaled_sum_to_half_bits((sa ? sa[batch * M + m] : 1.0f) * sbn, acc[m]);
    }
}

}  // namespace

hipError_t launch_bmm_s8(const int8_t *A, const int8_t *B, const float *sa, const float *sb, uint16_t *out, int32_t *acc_out,
                         int batch, int M, int N, int K, hipStream_t st)
{
    if (M <= 16) {
        int lpr_log2 = 0;
        while (lpr_log2 < 6 && (16 << lpr_log2) < K) ++lpr_log2;
        const int rows = 256 >> lpr_log2;
        const dim3 g((N + rows - 1) / rows, batch), b(256);
#define DGQ_ROWS(MT)                                                                                                  \
    do {                                                                                                              \
        if (acc_out)                                                                                                  \
            hipLaunchKernelGGL((bmm_s8_rows_kernel<MT, true>), g, b, 0, st, A, B, sa, sb, out, acc_out, M, N, K, lpr_log2); \
        else                                                                                                          \
            hipLaunchKernelGGL((bmm_s8_rows_kernel<MT, false>), g, b, 0, st, A, B, sa, sb, out, acc_out, M, N, K, lpr_log2); \
    } while (0)
        if (M == 1)
            DGQ_ROWS(1);
        else if (M <= 4)
            DGQ_ROWS(4);
        else
            DGQ_ROWS(16);
#undef DGQ_ROWS
        return hipGetLastError();
    }
    const dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM, batch), block(256);
    if (K > BK) {
        if (acc_out)
            hipLaunchKernelGGL((bmm_s8_kernel<true, true>), grid, block, 0, st, A, B, sa, sb, out, acc_out, M, N, K);
        else
            hipLaunchKernelGGL((bmm_s8_kernel<false, true>), grid, block, 0, st, A, B, sa, sb, out, acc_out, M, N, K);
    } else if (acc_out) {
        hipLaunchKernelGGL((bmm_s8_kernel<true, false>), grid, block, 0, st, A, B, sa, sb, out, acc_out, M, N, K);
    } else {
        hipLaunchKernelGGL((bmm_s8_kernel<false, false>), grid, block, 0, st, A, B, sa, sb, out, acc_out, M, N, K);
    }
    return hipGetLastError();
}

}  // namespace dgq
