// Tiled A8W4 linear for prefill-size M, bound by the INT8 matrix cores.
//
//   - Workgroup tile 128 tokens x 256 output channels, K walked in stages of 128; two
//     workgroups share a CU.  The four wavefronts split the output channels (64 each), so
//     every packed weight is expanded to INT8 exactly once per workgroup.
//   - Weights never touch LDS: each lane loads 16-byte cells of qweight straight into VGPRs
//     (a cell = 32 consecutive k of one column) two stages ahead of their use, expands them
//     with the group scale (second line of Eq. 2) and feeds them as the B operand of
//     v_mfma_i32_32x32x32_i8.
//   - The INT8 activation tile goes from global memory directly into a three-stage LDS ring
//     (global_load_lds_dwordx4, no registers in between), two stages ahead.  A row is 128
//     bytes = eight 16-byte units; unit u of row r is stored at unit u ^ ((r/2) % 8), so that
//     the 128-bit reads of sixteen consecutive rows (one read phase) fall on sixteen different
//     16-byte slots of the 256-byte bank line.  Lane (kb, i) reads as the A
//     operand the same k that the weight cell of lane (kb, j) holds.
//   - INT32 accumulation over all of K in AGPRs (third line of Eq. 2), then the scale
//     epilogue (first line of Eq. 2) and one rounding to fp16.
//   - Workgroups are numbered so that each XCD (workgroup id modulo 8) walks a contiguous
//     range of tiles, M fastest: the tiles resident on one XCD share weight columns in
//     that XCD's L2.
#include "dgq_device.hpp"

namespace dgq {
namespace {

constexpr int BM = 128;
constexpr int BN = 256;
constexpr int BK = 128;
constexpr int kStages = 3;
constexpr int kThreads = 256;

typedef __attribute__((address_space(3))) void *lptr_t;

// All global loads of the main loop are written as inline assembly, and all waiting for them
// is explicit (one s_waitcnt vmcnt(N) + barrier at the top of each stage).
//
// Why: the stage prefetch runs two stages ahead, both for weights (into registers) and for
// activations (straight into LDS).  The compiler makes every LDS read that follows a
// direct-to-LDS load it knows about wait for ALL outstanding vector loads (vmcnt(0)), which
// would serialise the prefetch behind the current stage.  With the loads invisible to its
// bookkeeping, the only waits are the ones written here, and they rely on vector loads
// completing in issue order: "at most N outstanding" means everything but the N youngest
// has landed.
typedef unsigned v4u __attribute__((ext_vector_type(4)));

// One wavefront copies 1 KiB from global memory straight into LDS: lane l's 16 bytes at `src`
// land at LDS byte address lds_base + 16*l (lds_base is wavefront-uniform and goes through M0).
__device__ __forceinline__ void lds_dma_1k(const void *src, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(src), "s"(lds_base)
                 : "memory", "m0");
}
__device__ __forceinline__ v4u load_b128_async(const void *src)
{
    v4u r;
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(r) : "v"(src) : "memory");
    return r;
}
__device__ __forceinline__ v4u load_b128_async_512(const void *src)
{
    v4u r;
    asm volatile("global_load_dwordx4 %0, %1, off offset:512" : "=v"(r) : "v"(src) : "memory");
    return r;
}
__device__ __forceinline__ uint32_t load_b32_async(const void *src)
{
    uint32_t r;
    asm volatile("global_load_dword %0, %1, off" : "=v"(r) : "v"(src) : "memory");
    return r;
}
// After the explicit wait: ties the registers of an asynchronously loaded set to this point, so
// that nothing that uses them can be scheduled above the wait and the registers stay reserved
// for the load until then.  EVERY register written by load_*_async must pass through here after
// the wait that covers it, also when its value is never used.
__device__ __forceinline__ void arrive(v4u &a, v4u &b, v4u &c, v4u &d, uint32_t &e, uint32_t &f)
{
    asm volatile("" : "+v"(a), "+v"(b), "+v"(c), "+v"(d), "+v"(e), "+v"(f));
}

template <int G, bool ACC>
__global__ __launch_bounds__(kThreads, 2) void linear_tiled_kernel(LinearArgs a, int tiles_m, int tiles_n)
{
    __shared__ __attribute__((aligned(1024))) int8_t lds_a[kStages][BM * BK];
#define DGQ_LDS(P) (lds_a[P])

    const int T = tiles_m * tiles_n;
    const int per_xcd = (T + 7) >> 3;
    const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile >= T) return;
    const int m0 = (tile % tiles_m) * BM;
    const int n0 = (tile / tiles_m) * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kb = lane >> 5;
    const int li = lane & 31;
    const int steps = a.K >> 7;
    const int gqn = ((a.K / G) + 3) >> 2;

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
    // ---- activation tile: each wavefront moves four 1 KiB pieces (8 rows) per stage --------
    // lane l of piece q lands at LDS row r = (wave*4+q)*8 + l/8, stored unit l%8, which is
    // the place of global unit (l%8) ^ ((r/2)%8).
    const int8_t *gp[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int r = (wave * 4 + q) * 8 + (lane >> 3);
        int m = m0 + r;
        if (m >= a.M) m = a.M - 1;  // ragged M: duplicate the last row, never store it
        gp[q] = a.xq + (size_t)m * a.K + (((lane & 7) ^ ((r >> 1) & 7)) << 4);
    }

    // LDS byte address of this wavefront's first piece in stage buffer 0
    const uint32_t lds_base = (uint32_t)(size_t)(lptr_t)&lds_a[0][0] + wave * 4096;

    v16i acc[4][2];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int nj = 0; nj < 2; ++nj)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][nj][r] = 0;

    v4u bq[kStages][2][2];    // [stage % 3][column tile][k half]
    uint32_t sw[kStages][2];  // [stage % 3][column tile]: four group scales of this lane's column

#define DGQ_LOAD_B(P, S)                                                   \
    do {                                                                   \
        const int s_ = (S);                                                \
        const int gq_ = ((G == 128) ? s_ : 2 * s_) >> 2;                   \
        _Pragma("unroll") for (int nj = 0; nj < 2; ++nj)                   \
        {                                                                  \
            bq[P][nj][0] = load_b128_async(bp[nj] + (size_t)s_ * 64);      \
            bq[P][nj][1] = load_b128_async_512(bp[nj] + (size_t)s_ * 64);  \
            sw[P][nj] = load_b32_async(sp[nj] + (size_t)gq_ * 16);         \
        }                                                                  \
    } while (0)
#define DGQ_LOAD_A(BUF, S)                                                                          \
    do {                                                                                            \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                               \
            lds_dma_1k(gp[q] + (size_t)(S) * BK, lds_base + (BUF) * (BM * BK) + q * 1024);          \
    } while (0)

    // per-lane LDS read offsets: row li of each 32-row block, units 2*kb + {0,1} (+4 for h=1)
    int a_off[2][2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int t = 0; t < 2; ++t) a_off[h][t] = li * BK + (((4 * h + 2 * kb + t) ^ ((li >> 1) & 7)) << 4);

    const int last = steps - 1;
    // prologue: stages 0 and 1 in flight
    DGQ_LOAD_B(0, 0);
    DGQ_LOAD_A(0, 0);
    DGQ_LOAD_B(1, last < 1 ? last : 1);
    DGQ_LOAD_A(1, last < 1 ? last : 1);

    // Stage s uses register set and LDS buffer s % 3 and refills set/buffer (s + 2) % 3, which
    // stage s - 1 used; the barrier at the top of stage s guarantees that every wavefront has
    // finished reading that buffer.
#define DGQ_STAGE(P, S)                                                                                 \
    do {                                                                                                \
        const int s_ = (S);                                                                             \
        /* stage s_ has landed once only the 10 loads of stage s_+1 (6 weight/scale loads and 4 */      \
        /* LDS copies per lane) are still outstanding                                          */      \
        __builtin_amdgcn_s_waitcnt(0x0F70 | 10);                                                        \
        __syncthreads();                                                                                \
        arrive(bq[P][0][0], bq[P][0][1], bq[P][1][0], bq[P][1][1], sw[P][0], sw[P][1]);                 \
        /* refill: stage s_+2 (past the end: re-read the last stage, unused) */                         \
        const int sn_ = s_ + 2 < steps ? s_ + 2 : last;                                                 \
        DGQ_LOAD_B((P + 2) % kStages, sn_);                                                             \
        DGQ_LOAD_A((P + 2) % kStages, sn_);                                                             \
        __builtin_amdgcn_sched_barrier(0); /* keep the prefetch at the top of the stage */              \
        const int8_t *la = &DGQ_LDS(P)[0];                                                                    \
        _Pragma("unroll") for (int h = 0; h < 2; ++h)                                                   \
        {                                                                                               \
            const int gi = (G == 128) ? s_ : 2 * s_ + h;                                                \
            v4i bf[2][2];                                                                               \
            _Pragma("unroll") for (int nj = 0; nj < 2; ++nj)                                            \
            {                                                                                           \
                const GroupScale gs = make_group_scale((sw[P][nj] >> (8 * (gi & 3))) & 0xFFu);          \
                expand_cell(__builtin_bit_cast(uint4, bq[P][nj][h]), gs, bf[nj][0], bf[nj][1]);                                 \
            }                                                                                           \
            _Pragma("unroll") for (int t = 0; t < 2; ++t)                                               \
            {                                                                                           \
                _Pragma("unroll") for (int mi = 0; mi < 4; ++mi)                                        \
                {                                                                                       \
                    const v4i af = *reinterpret_cast<const v4i *>(la + mi * 32 * BK + a_off[h][t]);     \
                    _Pragma("unroll") for (int nj = 0; nj < 2; ++nj) acc[mi][nj] =                      \
                        __builtin_amdgcn_mfma_i32_32x32x32_i8(af, bf[nj][t], acc[mi][nj], 0, 0, 0);     \
                }                                                                                       \
            }                                                                                           \
        }                                                                                               \
        __builtin_amdgcn_sched_barrier(0);                                                              \
    } while (0)

    int s = 0;
    for (; s + 3 <= steps; s += 3) {
        DGQ_STAGE(0, s);
        DGQ_STAGE(1, s + 1);
        DGQ_STAGE(2, s + 2);
    }
    if (s < steps) DGQ_STAGE(0, s);
    if (s + 1 < steps) DGQ_STAGE(1, s + 1);
    // The re-reads issued by the last two stages are unused but still in flight.  Their
    // destination registers must stay reserved until they have landed: a register the compiler
    // considers dead could be handed to another value and then be overwritten by the late load.
    __builtin_amdgcn_s_waitcnt(0x0F70);
#pragma unroll
    for (int p = 0; p < kStages; ++p) arrive(bq[p][0][0], bq[p][0][1], bq[p][1][0], bq[p][1][1], sw[p][0], sw[p][1]);
#undef DGQ_STAGE
#undef DGQ_LDS
#undef DGQ_LOAD_A
#undef DGQ_LOAD_B

    // ---- epilogue ---------------------------------------------------------------------------
    // acc[mi][nj][r] of lane l: token m0 + mi*32 + 8*(r/4) + 4*(l/32) + r%4, column ncol[nj].
    __syncthreads();  // every wavefront is done with the LDS ring
    if (ACC) {
#pragma unroll
        for (int nj = 0; nj < 2; ++nj) {
            const int n = ncol[nj];
            if (n >= a.N) continue;
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = m0 + mi * 32 + 8 * (r >> 2) + 4 * kb + (r & 3);
                    if (m < a.M) a.acc_out[(size_t)m * a.N + n] = acc[mi][nj][r];
                }
        }
        return;
    }
    // fp16 path.  The token scales of the tile go through LDS, so that scaling 128 accumulators
    // per lane does not wait on global memory.  The scaled fp16 values are then transposed
    // through a per-wavefront LDS region (64 tokens x 64 channels at a time) so that every lane
    // stores 16 contiguous bytes and eight lanes cover a whole 128-byte line of the output.
    float *lds_sx = reinterpret_cast<float *>(&lds_a[0][0]);
    unsigned short *lds_t = reinterpret_cast<unsigned short *>(&lds_a[0][0] + 1024 + wave * 8192);
    if (tid < BM) lds_sx[tid] = (m0 + tid < a.M) ? a.sx[m0 + tid] : 0.0f;
    float s1n[2];
#pragma unroll
    for (int nj = 0; nj < 2; ++nj) s1n[nj] = ncol[nj] < a.N ? a.s1[ncol[nj]] : 0.0f;
    __syncthreads();
    const int nw0 = n0 + wave * 64;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
#pragma unroll
        for (int mh = 0; mh < 2; ++mh) {
            const int mi = half * 2 + mh;
#pragma unroll
            for (int nj = 0; nj < 2; ++nj)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = mh * 32 + 8 * (r >> 2) + 4 * kb + (r & 3);
                    const float sc = lds_sx[half * 64 + row] * s1n[nj];
                    const _Float16 hv = (_Float16)(sc * (float)acc[mi][nj][r]);
                    lds_t[row * 64 + nj * 32 + li] = __builtin_bit_cast(unsigned short, hv);
                }
        }
        // 64 rows x 128 bytes: lane l takes 16-byte chunk l%8 of rows l/8, l/8 + 8, ...
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int row = j * 8 + (lane >> 3);
            const int m = m0 + half * 64 + row;
            const int n = nw0 + (lane & 7) * 8;
            const uint4 v = *reinterpret_cast<const uint4 *>(&lds_t[row * 64 + (lane & 7) * 8]);
            if (m < a.M && n < a.N) *reinterpret_cast<uint4 *>(&a.out[(size_t)m * a.N + n]) = v;
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
