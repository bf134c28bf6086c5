// Tiled A8W4 linear for prefill-size M, bound by the INT8 matrix cores.
//
//   - Workgroup tile 128 tokens x 256 output channels, K walked in stages of 128.
//     The four wavefronts split the output channels (64 each), so every packed weight is
//     expanded to INT8 exactly once per workgroup.
//   - Weights never touch LDS: each lane loads 16-byte cells of qweight straight into VGPRs
//     (a cell = 32 consecutive k of one column), expands them with the group scale
//     (second line of Eq. 2) and feeds them as the B operand of v_mfma_i32_32x32x32_i8.
//   - The INT8 activation tile is staged through LDS (double buffered, rows padded by 16
//     bytes so that 128-bit reads of 8 consecutive rows hit distinct banks) and read as the
//     A operand; lane (kb, i) reads the same k the weight cell of lane (kb, j) holds.
//   - INT32 accumulation over all of K (third line of Eq. 2), then the scale epilogue
//     (first line of Eq. 2) and one rounding to fp16.
//   - Workgroups are numbered so that each XCD (workgroup id modulo 8) walks a contiguous
//     range of tiles, M fastest: the tiles resident on one XCD share weight columns in
//     that XCD's L2.
#include "dgq_device.hpp"

namespace dgq {
namespace {

constexpr int BM = 128;
constexpr int BN = 256;
constexpr int BK = 128;
constexpr int LDA = BK + 16;
constexpr int kThreads = 256;

template <int G, bool ACC>
__global__ __launch_bounds__(kThreads) void linear_tiled_kernel(LinearArgs a, int tiles_m, int tiles_n)
{
    __shared__ __attribute__((aligned(16))) int8_t lds_a[2][BM * LDA];

    const int T = tiles_m * tiles_n;
    const int per_xcd = (T + 7) >> 3;
    const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile >= T) return;
    const int m0 = (tile % tiles_m) * BM;
    const int n0 = (tile / tiles_m) * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int kb = lane >> 5;
    const int li = lane & 31;
    const int steps = a.K >> 7;
    const int ng = a.K / G;
    const int gqn = (ng + 3) >> 2;

    // ---- weight stream: two 32-column tiles per wavefront -------------------------------
    const uint4 *bp[2];
    const uint32_t *sp[2];
    int ncol[2];
#pragma unroll
    for (int nj = 0; nj < 2; ++nj) {
        int n = n0 + wave * 64 + nj * 32 + li;
        ncol[nj] = n;
        if (n >= a.N) n = a.N - 1;  // ragged N: read a valid column, never store it
        bp[nj] = a.qweight + (size_t)(n >> 4) * steps * 64 + kb * 16 + (n & 15);
        sp[nj] = a.scales + (size_t)(n >> 4) * gqn * 16 + (n & 15);
    }
    // ---- activation tile: thread copies four 16-byte units per stage ----------------------
    const int unit = tid & 7;
    const uint4 *gp[4];
    int lds_off[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int r = (tid >> 3) + 32 * q;
        int m = m0 + r;
        if (m >= a.M) m = a.M - 1;  // ragged M: duplicate the last row, never store it
        gp[q] = reinterpret_cast<const uint4 *>(a.xq + (size_t)m * a.K + unit * 16);
        lds_off[q] = r * LDA + unit * 16;
    }

    v16i acc[4][2];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int nj = 0; nj < 2; ++nj)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][nj][r] = 0;

    uint4 ga[4];     // activation units in flight from global memory to LDS
    uint4 bq[2][2];  // weight cells of the next stage: [column tile][k half]
    uint32_t sw[2];  // four group scales of each of this lane's two columns

#define DGQ_LOAD_STAGE(S)                                                                   \
    do {                                                                                    \
        const int s_ = (S);                                                                 \
        _Pragma("unroll") for (int q = 0; q < 4; ++q) ga[q] = gp[q][(size_t)s_ * (BK / 16)]; \
        const int gq_ = ((G == 128) ? s_ : 2 * s_) >> 2;                                    \
        _Pragma("unroll") for (int nj = 0; nj < 2; ++nj)                                    \
        {                                                                                   \
            bq[nj][0] = bp[nj][(size_t)s_ * 64];                                            \
            bq[nj][1] = bp[nj][(size_t)s_ * 64 + 32];                                       \
            sw[nj] = sp[nj][(size_t)gq_ * 16];                                              \
        }                                                                                   \
    } while (0)
#define DGQ_STORE_A(BUF)                                                                   \
    do {                                                                                    \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                       \
            *reinterpret_cast<uint4 *>(&lds_a[(BUF)][lds_off[q]]) = ga[q];                  \
    } while (0)

    DGQ_LOAD_STAGE(0);
    DGQ_STORE_A(0);
    __syncthreads();

    const int a_lane_off = li * LDA + kb * 32;
    for (int s = 0; s < steps; ++s) {
        const int cur = s & 1;
        uint4 cq[2][2];
        uint32_t csw[2];
#pragma unroll
        for (int nj = 0; nj < 2; ++nj) {
            cq[nj][0] = bq[nj][0];
            cq[nj][1] = bq[nj][1];
            csw[nj] = sw[nj];
        }
        // Prefetch the next stage; the last iteration re-reads its own stage (unused).
        DGQ_LOAD_STAGE(s + 1 < steps ? s + 1 : s);

        const int8_t *la = &lds_a[cur][a_lane_off];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int gi = (G == 128) ? s : 2 * s + h;
            v4i bf[2][2];
#pragma unroll
            for (int nj = 0; nj < 2; ++nj) {
                const GroupScale gs = make_group_scale((csw[nj] >> (8 * (gi & 3))) & 0xFFu);
                expand_cell(cq[nj][h], gs, bf[nj][0], bf[nj][1]);
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int mi = 0; mi < 4; ++mi) {
                    const v4i af = *reinterpret_cast<const v4i *>(la + mi * 32 * LDA + h * 64 + t * 16);
#pragma unroll
                    for (int nj = 0; nj < 2; ++nj)
                        acc[mi][nj] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af, bf[nj][t], acc[mi][nj], 0, 0, 0);
                }
            }
        }
        // The other buffer was last read before the barrier that ended the previous
        // iteration, so it can be overwritten now.
        DGQ_STORE_A(cur ^ 1);
        __syncthreads();
    }
#undef DGQ_LOAD_STAGE
#undef DGQ_STORE_A

    // acc[mi][nj][r] of lane l: token m0 + mi*32 + 8*(r/4) + 4*(l/32) + r%4, column ncol[nj].
#pragma unroll
    for (int nj = 0; nj < 2; ++nj) {
        const int n = ncol[nj];
        if (n >= a.N) continue;
        float s1n = 0.0f;
        if (!ACC) s1n = a.s1[n];
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + mi * 32 + 8 * (r >> 2) + 4 * kb + (r & 3);
                if (m < a.M) {
                    if (ACC) {
                        a.acc_out[(size_t)m * a.N + n] = acc[mi][nj][r];
                    } else {
                        const float sc = a.sx[m] * s1n;
                        const _Float16 hv = (_Float16)(sc * (float)acc[mi][nj][r]);
                        a.out[(size_t)m * a.N + n] = __builtin_bit_cast(unsigned short, hv);
                    }
                }
            }
        }
    }
}

}  // namespace

hipError_t launch_linear_tiled(const LinearArgs &a, hipStream_t st)
{
    const int tiles_m = (a.M + BM - 1) / BM;
    const int tiles_n = (a.N + BN - 1) / BN;
    const long long T = (long long)tiles_m * tiles_n;
    const long long blocks = ((T + 7) / 8) * 8;
    if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)blocks), block(kThreads);
    if (a.group == 128) {
        if (a.acc_out)
            hipLaunchKernelGGL((linear_tiled_kernel<128, true>), grid, block, 0, st, a, tiles_m, tiles_n);
        else
            hipLaunchKernelGGL((linear_tiled_kernel<128, false>), grid, block, 0, st, a, tiles_m, tiles_n);
    } else {
        if (a.acc_out)
            hipLaunchKernelGGL((linear_tiled_kernel<64, true>), grid, block, 0, st, a, tiles_m, tiles_n);
        else
            hipLaunchKernelGGL((linear_tiled_kernel<64, false>), grid, block, 0, st, a, tiles_m, tiles_n);
    }
    return hipGetLastError();
}

}  // namespace dgq
