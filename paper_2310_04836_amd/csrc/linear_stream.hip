// Weight-streaming A8W4 linear for M <= 64, the simplest of the three GEMM kernels.  It is not
// chosen by M any more (the decode kernel serves M <= 16 and the tiled kernel everything above:
// this kernel re-reads the activations at every step and is bound by that L2 traffic for
// M > 16); it stays selectable as an independently written check of the other two, for the
// signed-nibble operands only.
//
//   - One workgroup owns one tile of 16 output channels; its W wavefronts split K between
//     them (split-K inside the workgroup) and combine their INT32 partial sums through LDS,
//     which is exact because integer addition is associative.
//   - Per step a wavefront reads one contiguous 1 KiB chunk of qweight (16 columns x 128 k,
//     one 128-bit load per lane), expands it in registers to two INT8 MFMA operands
//     (second line of Eq. 2), and issues two v_mfma_i32_16x16x64_i8 per 16-token tile
//     (third line of Eq. 2).  D steps of loads are kept in flight per wavefront.
//   - Activations come straight from global memory (they are tiny and cache resident):
//     lane (kb, i) reads the 32 bytes xq[i][128 s + 32 kb ...], which are exactly the k the
//     weight cell of lane (kb, j) holds, so both MFMA operands agree on the k of every byte.
//     Token rows beyond M re-read the last valid row; an output row depends only on its own
//     operand row, and those rows are never stored.
//   - The epilogue applies sx[m] * s1[n] (first line of Eq. 2) and rounds once to fp16.
#include "dgq_device.hpp"

namespace dgq {
namespace {

template <int MT>
struct Slot {
    uint4 q;          // one weight cell
    uint4 x[MT][2];   // 32 activation bytes per 16-token tile
    uint32_t sw;      // four consecutive group scales of this lane's column
};

template <int MT, int G, int W, int D, bool ACC>
__global__ __launch_bounds__(W * 64) void linear_stream_kernel(LinearArgs a)
{
    __shared__ int red[W * MT * 4 * 64];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ct = blockIdx.x;
    const int j = lane & 15;
    const int kb = lane >> 4;
    const int steps = a.K >> 7;
    const int sb = (steps * wave) / W;
    const int se = (steps * (wave + 1)) / W;
    const int gqn = ((a.K / G) + 3) >> 2;

    const uint4 *bp = a.qweight + (size_t)ct * steps * 64 + lane;
    const uint32_t *sp = a.scales + (size_t)ct * gqn * 16 + j;
    const uint4 *ap[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        int m = t * 16 + j;
        m = m < a.M ? m : a.M - 1;
        ap[t] = reinterpret_cast<const uint4 *>(a.xq + (size_t)m * a.K + kb * 32);
    }

    v4i acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[t] = v4i{0, 0, 0, 0};

    auto group_of = [&](int s) { return (G == 128) ? s : 2 * s + (kb >> 1); };
    auto load = [&](Slot<MT> &sl, int s) {
        s = s < se ? s : se - 1;  // past the end: re-read the last step, result unused
        sl.q = bp[(size_t)s * 64];
        sl.sw = sp[(size_t)(group_of(s) >> 2) * 16];
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            sl.x[t][0] = ap[t][(size_t)s * 8];
            sl.x[t][1] = ap[t][(size_t)s * 8 + 1];
        }
    };
    auto compute = [&](const Slot<MT> &sl, int s) {
        const GroupScale gs = make_group_scale((sl.sw >> (8 * (group_of(s) & 3))) & 0xFFu, 8u);
        v4i b0, b1;
        expand_cell(sl.q, gs, b0, b1);
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(v4i, sl.x[t][0]), b0, acc[t], 0, 0, 0);
            acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(v4i, sl.x[t][1]), b1, acc[t], 0, 0, 0);
        }
    };

    if (sb < se) {
        Slot<MT> slot[D];
#pragma unroll
        for (int d = 0; d < D; ++d) load(slot[d], sb + d);
        int s = sb;
        for (; s + D <= se; s += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                compute(slot[d], s + d);
                load(slot[d], s + D + d);
                // keep the refill here: a rolling window of D steps of loads in flight
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (s + d < se) compute(slot[d], s + d);
    }

    // acc[t][r] of lane l is the sum for token t*16 + 4*(l/16) + r and column ct*16 + l%16.
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[((wave * MT + t) * 4 + r) * 64 + lane] = acc[t][r];
    __syncthreads();

    for (int idx = threadIdx.x; idx < MT * 256; idx += W * 64) {
        const int t = idx >> 8;
        const int r = (idx >> 6) & 3;
        const int l = idx & 63;
        int sum = 0;
#pragma unroll
        for (int w = 0; w < W; ++w) sum += red[((w * MT + t) * 4 + r) * 64 + l];
        const int m = t * 16 + 4 * (l >> 4) + r;
        const int n = ct * 16 + (l & 15);
        if (m < a.M) {
            if (ACC) {
                a.acc_out[(size_t)m * a.N + n] = sum;
            } else {
                const float sc = a.sx[m] * a.s1[n];
                a.out[(size_t)m * a.N + n] = scaled_sum_to_half_bits(sc, sum);
            }
        }
    }
}

template <int MT, int G, int W, int D>
hipError_t launch_wd(const LinearArgs &a, hipStream_t st)
{
    dim3 grid(a.N / 16), block(W * 64);
    if (a.acc_out)
        hipLaunchKernelGGL((linear_stream_kernel<MT, G, W, D, true>), grid, block, 0, st, a);
    else
        hipLaunchKernelGGL((linear_stream_kernel<MT, G, W, D, false>), grid, block, 0, st, a);
    return hipGetLastError();
}

template <int MT, int G, int W>
hipError_t launch_w(const LinearArgs &a, int d, hipStream_t st)
{
    if constexpr (MT <= 2)
        if (d == 4) return launch_wd<MT, G, W, 4>(a, st);
    if (d >= 2) return launch_wd<MT, G, W, 2>(a, st);
    return launch_wd<MT, G, W, 1>(a, st);
}

template <int MT, int G>
hipError_t launch_mt(const LinearArgs &a, const StreamPlan &p, hipStream_t st)
{
    if constexpr (MT < 4)
        if (p.waves == 16) return launch_w<MT, G, 16>(a, p.depth, st);
    if (p.waves == 8) return launch_w<MT, G, 8>(a, p.depth, st);
    return launch_w<MT, G, 4>(a, p.depth, st);
}

template <int G>
hipError_t launch_g(const LinearArgs &a, const StreamPlan &p, hipStream_t st)
{
    if (p.mtiles == 1) return launch_mt<1, G>(a, p, st);
    if (p.mtiles == 2) return launch_mt<2, G>(a, p, st);
    return launch_mt<4, G>(a, p, st);
}

}  // namespace

StreamPlan stream_plan(int M, int N, int K)
{
    StreamPlan p;
    p.mtiles = M <= 16 ? 1 : (M <= 32 ? 2 : 4);
    // Enough wavefronts to keep every CU streaming (256 CUs x 16 wavefront slots); more
    // K-splitting only while each wavefront still has a couple of steps.
    const int tiles = N / 16;
    const int steps = K / 128;
    int w = 16;
    while (w > 4 && (tiles * w > 8192 || steps / w < 2)) w >>= 1;
    if (p.mtiles == 4 && w > 8) w = 8;  // LDS reduction buffer is waves * mtiles KiB
    p.waves = w;
    // loads in flight per wavefront: as many steps as it has, up to 4 (2 for wide token tiles)
    const int per_wave = steps / w;
    p.depth = (p.mtiles <= 2 && per_wave >= 4) ? 4 : (per_wave >= 2 ? 2 : 1);
    return p;
}

hipError_t launch_linear_stream(const LinearArgs &a, hipStream_t st)
{
    if (a.M > kStreamMaxM) return hipErrorInvalidValue;
    const StreamPlan p = stream_plan(a.M, a.N, a.K);
    return a.group == 128 ? launch_g<128>(a, p, st) : launch_g<64>(a, p, st);
}

}  // namespace dgq
