// Tiled A8W4 linear for M > 16: bound by the INT8 matrix cores at prefill sizes, by the weight
// stream up to M = 64.
//
//   - Workgroup tile (32*MI) tokens x (64*NW) output channels: 128 x 256 (four wavefronts, two
//     workgroups per CU) by default, 128 x 512 or 64 x 256 where the plan says so; K walked in
//     stages of 128.  The wavefronts split the output channels (64 each), so every packed
//     weight is expanded to INT8 exactly once per workgroup.
//   - Weights never touch LDS: each lane loads 16-byte cells of qweight straight into VGPRs
//     (a cell = 32 consecutive k of one column) ST - 1 = 2 stages ahead of their use, expands
//     them with the group scale (second line
//     of Eq. 2) and feeds them as the B operand of v_mfma_i32_32x32x32_i8.
//   - The INT8 activation tile goes from global memory directly into an ST-stage LDS ring
//     (global_load_lds_dwordx4, no registers in between), as far ahead.  A row is 128
//     bytes = eight 16-byte units; unit u of row r is stored at unit u ^ ((r/2) % 8), so that
//     the 128-bit reads of sixteen consecutive rows (one read phase) fall on sixteen different
//     16-byte slots of the 256-byte bank line.  Lane (kb, i) reads as the A
//     operand the same k that the weight cell of lane (kb, j) holds.
//   - INT32 accumulation over all of K (third line of Eq. 2), then the scale epilogue (first
//     line of Eq. 2) and one rounding to fp16.  When several workgroups split the K of one tile,
//     each leaves its INT32 partial sums in the workspace and counts itself in on the tile's
//     counter; the workgroup that arrives last adds the others' sums to its own (integer
//     addition: any order gives the same bits) and runs the epilogue.  Nobody waits for anybody,
//     so the scheme cannot hang whatever the number of resident workgroups.
//   - Workgroups are numbered so that each XCD (workgroup id modulo 8) walks a contiguous
//     range of tiles, ordered in bands of eight column tiles: the 64 workgroups resident on
//     one XCD cover about 8 x 8 tiles and share their operands in that XCD's L2.
#include "dgq_device.hpp"

#include <cmath>
#include <cstdio>

namespace dgq {
namespace {

constexpr int BK = 128;

// s_waitcnt immediate: at most n vector loads outstanding; LDS/scalar counter either ignored or
// waited down to zero.  (vmcnt is split over bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8.)
constexpr int wait_vm(int n, bool lgkm0) { return (n & 15) | ((n >> 4) << 14) | 0x0070 | (lgkm0 ? 0 : 0x0F00); }

typedef __attribute__((address_space(3))) void *lptr_t;

// All global loads of the main loop are written as inline assembly, and all waiting for them
// is explicit (one s_waitcnt vmcnt(N) + barrier per stage).
//
// Why: the stage prefetch runs several stages ahead, both for weights (into registers) and for
// activations (straight into LDS).  The compiler makes every LDS read that follows a
// direct-to-LDS load it knows about wait for ALL outstanding vector loads (vmcnt(0)), which
// would serialise the prefetch behind the current stage.  With the loads invisible to its
// bookkeeping, the only waits are the ones written here, and they rely on vector loads
// completing in issue order: "at most N outstanding" means everything but the N youngest
// has landed.
typedef unsigned v4u __attribute__((ext_vector_type(4)));

// Addresses are a wavefront-uniform 64-bit base (SGPR pair, advanced per stage with scalar
// arithmetic) plus a per-lane 32-bit byte offset that never changes, so the main loop computes
// no vector addresses at all.

// One wavefront copies 1 KiB from global memory straight into LDS: lane l's 16 bytes at
// base + off land at LDS byte address lds_base + 16*l (lds_base is uniform and goes through M0).
__device__ __forceinline__ void lds_dma_1k(const void *base, uint32_t off, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(off), "s"(base), "s"(lds_base)
                 : "memory", "m0");
}
__device__ __forceinline__ v4u load_b128_async(const void *base, uint32_t off)
{
    v4u r;
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(r) : "v"(off), "s"(base) : "memory");
    return r;
}
__device__ __forceinline__ v4u load_b128_async_512(const void *base, uint32_t off)
{
    v4u r;
    asm volatile("global_load_dwordx4 %0, %1, %2 offset:512" : "=v"(r) : "v"(off), "s"(base) : "memory");
    return r;
}
__device__ __forceinline__ uint32_t load_b32_async(const void *base, uint32_t off)
{
    uint32_t r;
    asm volatile("global_load_dword %0, %1, %2" : "=v"(r) : "v"(off), "s"(base) : "memory");
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

// NW wavefronts per workgroup, each owning 64 output channels of the (32*MI) x (64*NW) tile;
// ST stages of operands in flight or in use.  ksplit workgroups share one tile, each walking its
// own part of K (see SplitK below).  ACC: the test hook, raw INT32 sums to a.acc_out.
// ZP: the scale words hold (S2, ZP) pairs instead of S2 bytes; a compile-time choice, so that the
// signed-nibble form pays nothing for the general one.
// Workspace of a K split: one counter per tile (zero before the launch, zero again after it),
// then for every tile and part a block of BM x BN INT32 partial sums in register order.
struct SplitK {
    int parts;           // workgroups per tile (1: no split, the pointers are unused)
    uint32_t *counters;  // [tiles]
    int32_t *partial;    // [tiles][parts][BM * BN]
};

// SPLIT is a compile-time choice so that the kernels without a K split carry none of its code.
// COLS: the launch covers a range of the output channels of a wider layer (rows of the output are
// a.ldo elements apart instead of a.N).
template <int G, int NW, int MI, int ST, bool ACC, bool ZP, bool SPLIT, bool COLS = false>
__device__ __forceinline__ void tiled_body(const LinearArgs &a, int tiles_m, int tiles_n, const SplitK &sk)
{
    const int ksplit = SPLIT ? sk.parts : 1;
    const int ldo = COLS ? a.ldo : a.N;
    constexpr int kStages = ST;
    constexpr int BM = 32 * MI;
    constexpr int BN = 64 * NW;
    constexpr int PPW = BM / (8 * NW);  // 1 KiB pieces of the activation tile each wavefront copies per stage
    constexpr int kLoadsPerStage = 6 + PPW;
    static_assert(MI == 2 || MI == 4, "two or four 32-token blocks");
    static_assert(ST >= 3 && ST <= 6 && PPW >= 1 && kLoadsPerStage <= 12, "loads are spread over 12 sub-chunks");
    static_assert((ST - 1) * kLoadsPerStage <= 63, "vmcnt counts to 63");
    static_assert(1024 + NW * 4096 <= ST * BM * BK, "the epilogue reuses the ring");

    __shared__ __attribute__((aligned(1024))) int8_t lds_a[kStages][BM * BK];

    const int T = tiles_m * tiles_n * ksplit;
    const int per_xcd = (T + 7) >> 3;
    const int work = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (work >= T) return;
    const int tile = work / ksplit;
    const int kpart = work - tile * ksplit;
    // Tiles are numbered in bands of eight column tiles: inside a band the column tile runs
    // fastest, then the token tile.  The 64 workgroups resident on an XCD then cover about
    // 8 x 8 tiles, the shape that needs the fewest operand bytes in that XCD's L2.
    const int band = tile / (8 * tiles_m);
    const int in_band = tile - band * (8 * tiles_m);
    const int band_w = tiles_n - band * 8 < 8 ? tiles_n - band * 8 : 8;
    const int m0 = (in_band / band_w) * BM;
    const int n0 = (band * 8 + in_band % band_w) * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kb = lane >> 5;
    const int li = lane & 31;
    const int steps = a.K >> 7;
    const ScaleForm sf = scale_form(ZP ? 1 : 0);  // scale words hold 4 groups (S2 bytes) or 2 (S2, ZP pairs)
    const int fsh = sf.fsh;
    const int gqn = ((a.K / G) + (1 << fsh) - 1) >> fsh;

    // ---- weight stream: two 32-column tiles per wavefront ------------------------------------
    // Per-lane byte offsets are relative to the tile's first 16-column block and first token
    // (at most 128 K bytes, whatever the size of the tensors); the tile's origin is part of the
    // 64-bit scalar base.
    const char *q_tile = reinterpret_cast<const char *>(a.qweight) + (size_t)(n0 >> 4) * steps * 1024;
    const char *s_tile = reinterpret_cast<const char *>(a.scales) + (size_t)(n0 >> 4) * gqn * 64;
    const char *x_tile = reinterpret_cast<const char *>(a.xq) + (size_t)m0 * a.K;
    uint32_t boff[2], soff[2];
    int ncol[2];
#pragma unroll
    for (int nj = 0; nj < 2; ++nj) {
        int n = n0 + wave * 64 + nj * 32 + li;
        ncol[nj] = n;
        if (n >= a.N) n = a.N - 1;  // ragged N: read a valid column (n0 <= n), never store it
        const int nr = n - n0;      // N and n0 are multiples of 16, so nr/16 counts whole blocks
        boff[nj] = ((uint32_t)(nr >> 4) * steps * 64 + kb * 16 + (nr & 15)) * 16u;
        soff[nj] = ((uint32_t)(nr >> 4) * gqn * 16 + (nr & 15)) * 4u;
    }
    // ---- activation tile: each wavefront moves PPW 1 KiB pieces (8 rows each) per stage ------
    // lane l of piece q lands at LDS row r = (wave*PPW+q)*8 + l/8, stored unit l%8, which is
    // the place of global unit (l%8) ^ ((r/2)%8).
    uint32_t goff[PPW];
#pragma unroll
    for (int q = 0; q < PPW; ++q) {
        const int r = (wave * PPW + q) * 8 + (lane >> 3);
        int m = m0 + r;
        if (m >= a.M) m = a.M - 1;  // ragged M: duplicate the last row (m0 <= m), never store it
        goff[q] = (uint32_t)(m - m0) * a.K + (((lane & 7) ^ ((r >> 1) & 7)) << 4);
    }

    // ---- epilogue operands, requested now -----------------------------------------------------
    // One token scale per thread (threads past the tile's tokens repeat a valid one) and the
    // channel scales of this lane's two columns.  Asked for here, in front of the first stage, they
    // cost three registers through the main loop; asked for after it they add a memory latency to
    // every tile, which shows where a workgroup has its CU to itself (64-token tiles: 1-5 % per
    // launch).  The 128-token tiles use all 256 registers a wavefront can have at two per SIMD and
    // gain nothing measurable, so they keep asking late.  These are the oldest vector loads, so the
    // first wait of the prologue covers them.
    constexpr bool kEarlyScales = !ACC && MI == 2;
    uint32_t ep_sx = 0, ep_s1[2] = {0, 0};
    if constexpr (kEarlyScales) {
        int mrow = m0 + (tid < BM ? tid : 0);
        if (mrow >= a.M) mrow = a.M - 1;
        ep_sx = load_b32_async(a.sx, (uint32_t)mrow * 4u);
#pragma unroll
        for (int nj = 0; nj < 2; ++nj) ep_s1[nj] = load_b32_async(a.s1, (uint32_t)(ncol[nj] < a.N ? ncol[nj] : a.N - 1) * 4u);
    }

    // LDS byte address of this wavefront's first piece in stage buffer 0
    const uint32_t lds_base = (uint32_t)(size_t)(lptr_t)&lds_a[0][0] + wave * PPW * 1024;

    // this workgroup's stages of K
    const int p0 = (steps * kpart) / ksplit;
    const int p1 = (steps * (kpart + 1)) / ksplit;

    v16i acc[MI][2];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int nj = 0; nj < 2; ++nj)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][nj][r] = 0;

    v4u bq[kStages][2][2];    // [stage % ST][column tile][k half]
    uint32_t sw[kStages][2];  // [stage % ST][column tile]: four group scales of this lane's column

    // The loads of one stage are 6 + PPW instructions per lane, always in
    // this order: weight cells and scales of the two column tiles, then the LDS copies.  Item I of
    // stage S, into register set / LDS buffer P:
#define DGQ_LOAD_ITEM(I, P, S)                                                                        \
    do {                                                                                              \
        const int ls_ = (S);                                                                          \
        const char *qb_ = q_tile + (size_t)ls_ * 1024;                                                \
        const char *sb_ = s_tile + (size_t)(((G == 128) ? ls_ : 2 * ls_) >> fsh) * 64;                \
        const char *xb_ = x_tile + (size_t)ls_ * BK;                                                  \
        if ((I) == 0) bq[P][0][0] = load_b128_async(qb_, boff[0]);                                    \
        else if ((I) == 1) bq[P][0][1] = load_b128_async_512(qb_, boff[0]);                           \
        else if ((I) == 2) sw[P][0] = load_b32_async(sb_, soff[0]);                                   \
        else if ((I) == 3) bq[P][1][0] = load_b128_async(qb_, boff[1]);                               \
        else if ((I) == 4) bq[P][1][1] = load_b128_async_512(qb_, boff[1]);                           \
        else if ((I) == 5) sw[P][1] = load_b32_async(sb_, soff[1]);                                   \
        else if ((I) < kLoadsPerStage)                                                                \
            lds_dma_1k(xb_, goff[((I) - 6) % PPW], lds_base + (P) * (BM * BK) + (((I) - 6) % PPW) * 1024); \
    } while (0)
#define DGQ_LOAD_STAGE(P, S)                                                                          \
    do {                                                                                              \
        _Pragma("unroll") for (int i_ = 0; i_ < kLoadsPerStage; ++i_) DGQ_LOAD_ITEM(i_, P, S);        \
    } while (0)
#define DGQ_ARRIVE(P) arrive(bq[P][0][0], bq[P][0][1], bq[P][1][0], bq[P][1][1], sw[P][0], sw[P][1])

    // per-lane LDS read offsets: row li of each 32-row block, units 2*kb + t (+4 for h = 1)
    int a_off[4];
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) a_off[g4] = li * BK + (((2 * g4 - (g4 & 1) + 2 * kb) ^ ((li >> 1) & 7)) << 4);

    // The 128 k of a stage are consumed in four groups (h, t) = (0,0), (0,1), (1,0), (1,1) of
    // 2*MI MFMAs each, and a group in four sub-chunks: two MFMAs (one 32-token block, both
    // column tiles) for MI = 4, one MFMA for MI = 2.  A wavefront issues in order, so anything that sits between two MFMAs for
    // longer than an MFMA runs (32 cycles) drains the matrix pipe.  Every sub-chunk therefore
    // carries an even share of the other work, all of it for LATER use: one LDS read and one
    // word (2 x 4 weights) of expansion for the same sub-chunk of the next group, into the
    // other half of two-deep register buffers, and at most one of the stage's global loads.
    v4i af[2][MI];  // [group parity][mi]
    v4i bf[2][2];  // [group parity][nj]
    GroupScale gsn[2];
    // (a group of 128 k is a whole stage, a group of 64 k half of one: new scales are needed at
    // k-group 0 and, for G = 64, at k-group 2)
#define DGQ_SCALES(PN, SN, GRPN)                                                                      \
    do {                                                                                              \
        if ((GRPN) == 0 || (G == 64 && (GRPN) == 2)) {                                                \
            const int gi_ = (G == 128) ? (SN) : 2 * (SN) + ((GRPN) >> 1);                             \
            const uint32_t sh_ = scale_entry_shift(gi_, sf);                                          \
            _Pragma("unroll") for (int nj = 0; nj < 2; ++nj) gsn[nj] = group_scale_at(sw[PN][nj], sh_, sf); \
        }                                                                                             \
    } while (0)
    // prepares piece C of group GRPN (stage set PN) into parity PARN
#define DGQ_PREP(PARN, C, PN, GRPN)                                                                   \
    do {                                                                                              \
        if ((C) < MI)                                                                                 \
            af[PARN][(C) % MI] = *reinterpret_cast<const v4i *>(&lds_a[PN][((C) % MI) * 32 * BK + a_off[GRPN]]); \
        _Pragma("unroll") for (int nj = 0; nj < 2; ++nj)                                              \
        {                                                                                             \
            const uint32_t w_ = bq[PN][nj][(GRPN) >> 1][C];                                           \
            bf[PARN][nj][C] = (int)scale_bytes((((GRPN) & 1) ? (w_ >> 4) : w_) & 0x0F0F0F0Fu, gsn[nj]); \
        }                                                                                             \
    } while (0)
    // sub-chunk C of a group with operand parity PAR: prepare piece C of the next group, the
    // MFMAs, optionally load item LI of stage LS into set LP
#define DGQ_SUB(PAR, C, PN, GRPN, LI, LP, LS)                                                         \
    do {                                                                                              \
        DGQ_PREP((PAR) ^ 1, C, PN, GRPN);                                                             \
        if (MI == 4) {                                                                                \
            acc[(C) % MI][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[PAR][(C) % MI], bf[PAR][0],   \
                                                                     acc[(C) % MI][0], 0, 0, 0);     \
            acc[(C) % MI][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[PAR][(C) % MI], bf[PAR][1],   \
                                                                     acc[(C) % MI][1], 0, 0, 0);     \
        } else {                                                                                      \
            acc[((C) >> 1) % MI][(C) & 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(                    \
                af[PAR][((C) >> 1) % MI], bf[PAR][(C) & 1], acc[((C) >> 1) % MI][(C) & 1], 0, 0, 0);  \
        }                                                                                             \
        DGQ_LOAD_ITEM(LI, LP, LS);                                                                    \
        __builtin_amdgcn_sched_barrier(0);                                                            \
    } while (0)
    // group with operand parity PAR whose sub-chunks carry load items LI0 .. LI0+3
#define DGQ_GROUP(PAR, PN, SN, GRPN, LI0, LP, LS)                                                     \
    do {                                                                                              \
        DGQ_SCALES(PN, SN, GRPN);                                                                     \
        DGQ_SUB(PAR, 0, PN, GRPN, (LI0) + 0, LP, LS);                                                 \
        DGQ_SUB(PAR, 1, PN, GRPN, (LI0) + 1, LP, LS);                                                 \
        DGQ_SUB(PAR, 2, PN, GRPN, (LI0) + 2, LP, LS);                                                 \
        DGQ_SUB(PAR, 3, PN, GRPN, (LI0) + 3, LP, LS);                                                 \
    } while (0)

    const int last = p1 - 1;
    // prologue: the first ST - 1 stages in flight (stages past the end re-read the last one,
    // unused); operands of the first group prepared
#pragma unroll
    for (int p = 0; p < kStages - 1; ++p) DGQ_LOAD_STAGE(p, p0 + p < last ? p0 + p : last);
    __builtin_amdgcn_s_waitcnt(wait_vm((kStages - 2) * kLoadsPerStage, false));  // the first stage has landed
    __syncthreads();
    DGQ_ARRIVE(0);
    if constexpr (kEarlyScales) asm volatile("" : "+v"(ep_sx), "+v"(ep_s1[0]), "+v"(ep_s1[1]));
    DGQ_SCALES(0, p0, 0);
#pragma unroll
    for (int c = 0; c < 4; ++c) DGQ_PREP(0, c, 0, 0);

    // The i-th stage of this workgroup uses register set and LDS buffer i % ST.  On entry
    // af[0] / bf[0] already hold the operands of its group 0: they were prepared during the last
    // group of the stage before, after that stage's barrier.  Groups 0-2 also issue the loads of
    // the stage ST - 1 ahead, one per sub-chunk, into the buffer of the stage before this one.
    // The barrier before group 3 says two things at once: the data of the next stage have landed
    // for every wavefront (only the loads of the ST - 2 stages after it are still outstanding),
    // and every wavefront has finished its LDS reads of this stage (lgkmcnt(0) precedes the
    // barrier), so the copies that the next stage issues into this buffer cannot overtake a reader.
#define DGQ_STAGE(P, S)                                                                               \
    do {                                                                                              \
        const int s_ = (S);                                                                           \
        const int s2_ = s_ + (kStages - 1) < p1 ? s_ + (kStages - 1) : last; /* past the end: unused */ \
        DGQ_GROUP(0, P, s_, 1, 0, (P + kStages - 1) % kStages, s2_);                                  \
        DGQ_GROUP(1, P, s_, 2, 4, (P + kStages - 1) % kStages, s2_);                                  \
        DGQ_GROUP(0, P, s_, 3, 8, (P + kStages - 1) % kStages, s2_);                                  \
        __builtin_amdgcn_s_waitcnt(wait_vm((kStages - 2) * kLoadsPerStage, true));                    \
        __syncthreads();                                                                              \
        DGQ_ARRIVE((P + 1) % kStages);                                                                \
        DGQ_GROUP(1, (P + 1) % kStages, s_ + 1, 0, 12, (P + kStages - 1) % kStages, s2_);             \
    } while (0)

    int s = p0;
    for (; s + kStages <= p1; s += kStages) {
        DGQ_STAGE(0, s);
        DGQ_STAGE(1, s + 1);
        DGQ_STAGE(2, s + 2);
        if constexpr (kStages > 3) DGQ_STAGE(3 % kStages, s + 3);
        if constexpr (kStages > 4) DGQ_STAGE(4 % kStages, s + 4);
        if constexpr (kStages > 5) DGQ_STAGE(5 % kStages, s + 5);
    }
    // the remaining 0 .. ST - 1 stages, nested so that no path runs stage i + 1 without stage i
    if (s < p1) {
        DGQ_STAGE(0, s);
        if (s + 1 < p1) {
            DGQ_STAGE(1, s + 1);
            if constexpr (kStages > 3) {
                if (s + 2 < p1) {
                    DGQ_STAGE(2, s + 2);
                    if constexpr (kStages > 4) {
                        if (s + 3 < p1) {
                            DGQ_STAGE(3 % kStages, s + 3);
                            if constexpr (kStages > 5) {
                                if (s + 4 < p1) DGQ_STAGE(4 % kStages, s + 4);
                            }
                        }
                    }
                }
            }
        }
    }
    // The re-reads issued by the last stages are unused but still in flight.  Their
    // destination registers must stay reserved until they have landed: a register the compiler
    // considers dead could be handed to another value and then be overwritten by the late load.
    __builtin_amdgcn_s_waitcnt(wait_vm(0, false));
#pragma unroll
    for (int p = 0; p < kStages; ++p) DGQ_ARRIVE(p);
#undef DGQ_STAGE
#undef DGQ_GROUP
#undef DGQ_SUB
#undef DGQ_PREP
#undef DGQ_SCALES
#undef DGQ_ARRIVE
#undef DGQ_LOAD_STAGE
#undef DGQ_LOAD_ITEM

    // ---- K split: the last workgroup of a tile to arrive adds up the parts ----------------------
    if constexpr (SPLIT) {
        // Block (tile, part) holds the sums in register order: pair j = (mi*2 + nj)*8 + r/2 of
        // wavefront w and lane l at 8-byte unit (w*MI*16 + j)*64 + l, so that every store and
        // load of a wavefront covers 512 bytes of contiguous memory.
        //
        // Stores and loads of partial sums are relaxed atomics of device scope: they go through to
        // (come from) the level of the memory system that all compute units share, and nothing else
        // in the caches is written back or invalidated for them.  Order between the sums and the
        // counter is kept by hand: a wavefront waits until its stores have completed (vmcnt(0))
        // before the barrier behind which the workgroup counts itself in, and the last arriver
        // issues its loads only after the counter's old value has come back.
        unsigned long long *blk = reinterpret_cast<unsigned long long *>(sk.partial + ((size_t)tile * ksplit + kpart) * (BM * BN)) +
                                  wave * (MI * 16) * 64 + lane;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int nj = 0; nj < 2; ++nj)
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const unsigned long long v = (uint32_t)acc[mi][nj][2 * q] | ((unsigned long long)(uint32_t)acc[mi][nj][2 * q + 1] << 32);
                    __hip_atomic_store(&blk[((mi * 2 + nj) * 8 + q) * 64], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
        __builtin_amdgcn_s_waitcnt(wait_vm(0, true));   // this wavefront's sums have reached memory
        __syncthreads();
        uint32_t *arrived = reinterpret_cast<uint32_t *>(&lds_a[0][0]);
        if (tid == 0) *arrived = __hip_atomic_fetch_add(&sk.counters[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (*arrived != (uint32_t)(ksplit - 1)) return;      // somebody else will finish this tile
        if (tid == 0) __hip_atomic_store(&sk.counters[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
        for (int p = 0; p < ksplit; ++p) {
            if (p == kpart) continue;
            const unsigned long long *ob = reinterpret_cast<const unsigned long long *>(sk.partial + ((size_t)tile * ksplit + p) * (BM * BN)) +
                                           wave * (MI * 16) * 64 + lane;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int nj = 0; nj < 2; ++nj)
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        const unsigned long long o = __hip_atomic_load(&ob[((mi * 2 + nj) * 8 + q) * 64], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        acc[mi][nj][2 * q] += (int)(uint32_t)o;
                        acc[mi][nj][2 * q + 1] += (int)(uint32_t)(o >> 32);
                    }
        }
    }

    // ---- epilogue ---------------------------------------------------------------------------
    // acc[mi][nj][r] of lane l: token m0 + mi*32 + 8*(r/4) + 4*(l/32) + r%4, column ncol[nj].
    __syncthreads();  // every wavefront is done with the LDS ring
    if (ACC) {
        int32_t *dst = a.acc_out;
#pragma unroll
        for (int nj = 0; nj < 2; ++nj) {
            const int n = ncol[nj];
            if (n >= a.N) continue;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = m0 + mi * 32 + 8 * (r >> 2) + 4 * kb + (r & 3);
                    if (m < a.M) dst[(size_t)m * ldo + n] = acc[mi][nj][r];
                }
        }
        return;
    }
    // fp16 path.  The token scales of the tile go through LDS, so that scaling 128 accumulators
    // per lane does not wait on global memory.  The scaled fp16 values are then transposed
    // through a per-wavefront LDS region (32 tokens x 64 channels at a time) so that every lane
    // stores 16 contiguous bytes and eight lanes cover a whole 128-byte line of the output.
    float *lds_sx = reinterpret_cast<float *>(&lds_a[0][0]);
    unsigned short *lds_t = reinterpret_cast<unsigned short *>(&lds_a[0][0] + 1024 + wave * 4096);
    if (tid < BM) {
        if constexpr (kEarlyScales) lds_sx[tid] = (m0 + tid < a.M) ? __builtin_bit_cast(float, ep_sx) : 0.0f;
        else lds_sx[tid] = (m0 + tid < a.M) ? a.sx[m0 + tid] : 0.0f;
    }
    float s1n[2];
#pragma unroll
    for (int nj = 0; nj < 2; ++nj) {
        if constexpr (kEarlyScales) s1n[nj] = ncol[nj] < a.N ? __builtin_bit_cast(float, ep_s1[nj]) : 0.0f;
        else s1n[nj] = ncol[nj] < a.N ? a.s1[ncol[nj]] : 0.0f;
    }
    __syncthreads();
    const int nw0 = n0 + wave * 64;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
        for (int nj = 0; nj < 2; ++nj)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 8 * (r >> 2) + 4 * kb + (r & 3);
                const float sc = lds_sx[mi * 32 + row] * s1n[nj];
                lds_t[row * 64 + nj * 32 + li] = scaled_sum_to_half_bits(sc, acc[mi][nj][r]);
            }
        // 32 rows x 128 bytes: lane l takes 16-byte chunk l%8 of rows l/8, l/8 + 8, ...
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = j * 8 + (lane >> 3);
            const int m = m0 + mi * 32 + row;
            const int n = nw0 + (lane & 7) * 8;
            const uint4 v = *reinterpret_cast<const uint4 *>(&lds_t[row * 64 + (lane & 7) * 8]);
            // streaming store: the output is written once and read by another kernel; this keeps it
            // from displacing the operands the other tiles still share in L2 (1-4 % per launch)
            if (m < a.M && n < a.N)
                __builtin_nontemporal_store(__builtin_bit_cast(v4i, v), reinterpret_cast<v4i *>(&a.out[(size_t)m * ldo + n]));
        }
    }
}

template <int G, int NW, int MI, int ST, bool ACC>
__global__ __launch_bounds__(64 * NW, 2) void linear_tiled_kernel(LinearArgs a, int tiles_m, int tiles_n)
{
    tiled_body<G, NW, MI, ST, ACC, false, false>(a, tiles_m, tiles_n, SplitK{1, nullptr, nullptr});
}
template <int G, int NW, int MI, int ST, bool ACC>
__global__ __launch_bounds__(64 * NW, 2) void linear_tiled_zp_kernel(LinearArgs a, int tiles_m, int tiles_n)
{
    tiled_body<G, NW, MI, ST, ACC, true, false>(a, tiles_m, tiles_n, SplitK{1, nullptr, nullptr});
}
// the same for a range of the output channels of a wider layer
template <int G, int NW, int MI, int ST, bool ACC>
__global__ __launch_bounds__(64 * NW, 2) void linear_tiled_cols_kernel(LinearArgs a, int tiles_m, int tiles_n)
{
    tiled_body<G, NW, MI, ST, ACC, false, false, true>(a, tiles_m, tiles_n, SplitK{1, nullptr, nullptr});
}
template <int G, int NW, int MI, int ST, bool ACC>
__global__ __launch_bounds__(64 * NW, 2) void linear_tiled_cols_zp_kernel(LinearArgs a, int tiles_m, int tiles_n)
{
    tiled_body<G, NW, MI, ST, ACC, true, false, true>(a, tiles_m, tiles_n, SplitK{1, nullptr, nullptr});
}
// the same with the K of every tile split over sk.parts workgroups
template <int G, int NW, int MI, int ST, bool ACC>
__global__ __launch_bounds__(64 * NW, 2) void linear_tiled_splitk_kernel(LinearArgs a, int tiles_m, int tiles_n, SplitK sk)
{
    tiled_body<G, NW, MI, ST, ACC, false, true>(a, tiles_m, tiles_n, sk);
}
template <int G, int NW, int MI, int ST, bool ACC>
__global__ __launch_bounds__(64 * NW, 2) void linear_tiled_splitk_zp_kernel(LinearArgs a, int tiles_m, int tiles_n, SplitK sk)
{
    tiled_body<G, NW, MI, ST, ACC, true, true>(a, tiles_m, tiles_n, sk);
}

}  // namespace

namespace {
// Predicted duration (us) of one launch: a small model fitted to a sweep of 728 timings over the
// LLaMA-7B/13B/65B layer shapes at M = 64 ... 2048 (root-mean-square error 12 %).  It is only
// used to compare a plan with its K split over several workgroups against the unsplit plan.
//   stage    0.585 us for a 128 x 256 tile alone on a CU, in proportion to the tile's MFMA work;
//            2.56 x that when two workgroups share the CU (they also share its clock budget);
//            +0.13 us for 64-token tiles (every weight is expanded for half as many MFMAs)
//   launch   5.9 us (launch, first loads, epilogue)
//   split    1.1 us per further part and 64 KiB of tile for the last workgroup's additions, and
//            0.34 us per MB of partial sums (they go through to memory)
//   and never faster than the weights, activations and outputs take at 3.9 TB/s
double predicted_us(int M, int N, int K, const TiledPlan &p, int cus)
{
    const int bm = 32 * p.mi, bn = 64 * p.nw;
    const double tiles = (double)((M + bm - 1) / bm) * ((N + bn - 1) / bn);
    const double wgs = tiles * p.ksplit;
    const double slots = (double)cus * (p.nw == 4 ? 2 : 1);
    const double rounds = ceil(wgs / slots);
    const double resident = (wgs < slots ? wgs : slots) / cus;
    const double shared = p.nw == 4 && resident > 1.0 ? resident : 1.0;
    const double work = p.mi * p.nw / 16.0;
    const double t_stage = 0.585 * work * (1.0 + 1.563 * (shared - 1.0)) + (p.mi == 2 ? 0.133 : 0.0);
    const int steps = K / 128;
    double t = 5.948 + rounds * ((steps + p.ksplit - 1) / p.ksplit) * t_stage;
    if (p.ksplit > 1)
        t += 1.125 * (p.ksplit - 1) * (bm * bn * 4 / 65536.0) + 0.337 * (wgs * bm * bn * 4 / 1e6);
    const double stream = ((double)K * N / 2 + (double)M * K * rounds + 2.0 * M * N) / 3.919e6;
    return t > stream ? t : stream;
}
}  // namespace

// The plan without a K split.
static TiledPlan tiled_base_plan(int M, int N, int cus)
{
    TiledPlan p;
    p.nw = 4, p.mi = 4, p.st = 3, p.ksplit = 1;
    const long long tiles_n = (N + 255) / 256;
    const long long tiles_64 = (long long)((M + 63) / 64) * tiles_n;
    const long long tiles_128 = (long long)((M + 127) / 128) * tiles_n;
    if (M <= 64 || tiles_64 <= cus) {
        // Even 64-token tiles leave every workgroup a CU of its own: twice as many SIMDs work as
        // with 128-token tiles.  (With more tiles than CUs the smaller tile loses: it expands
        // every weight twice as often.)
        p.mi = 2;
    } else {
        // Two workgroups of four wavefronts per CU overlap better than one of eight: the two
        // wavefronts that share a SIMD then wait at different barriers.  The wide tile (128 x 512,
        // eight wavefronts) moves a quarter less operand data per MAC, which pays when its grid
        // fills the CUs as evenly as the narrow one's: in whole rounds, or in one round that
        // reaches most of them while the narrow tiles also fit one round.
        const long long wide = (long long)((M + 127) / 128) * ((N + 511) / 512);
        if ((wide >= cus && wide % cus == 0) || (wide >= 160 && wide <= cus && tiles_128 <= 2 * cus)) p.nw = 8;
    }
    return p;
}

TiledPlan tiled_plan(int M, int N, int K)
{
    const int cus = cu_count();
    const int steps = K / 128;
    const TiledPlan p = tiled_base_plan(M, N, cus);
    const long long tiles_n = (N + 255) / 256;
    const long long tiles_64 = (long long)((M + 63) / 64) * tiles_n;
    const long long tiles_128 = (long long)((M + 127) / 128) * tiles_n;
    // K split over several workgroups per tile (the last to arrive adds up the parts): for shapes
    // whose tiles alone leave CUs idle.  64-token tiles in 2 to 8 parts (at most two workgroups per
    // CU), 128-token tiles in 2 to 4 parts (every part a CU to itself); at least four stages per
    // part; taken when the model above predicts more than 3 % gain over the unsplit plan.  The
    // partial sums of such a plan never exceed 2 * CUs * 64 KiB.
    double best_t = predicted_us(M, N, K, p, cus);
    const double bar = 0.97 * best_t;
    TiledPlan best = p;
    static const int kParts[] = {2, 3, 4, 6, 8};
    for (int mi = 2; mi <= 4; mi += 2) {
        if (mi == 4 && M <= 64) continue;
        const long long tiles = mi == 2 ? tiles_64 : tiles_128;
        for (int ks : kParts) {
            if (steps / ks < 4) break;
            if (ks > (mi == 2 ? 8 : 4) || tiles * ks > (mi == 4 ? cus : 2 * cus)) break;   // every part resident at once
            TiledPlan c;
            c.nw = 4, c.mi = mi, c.st = 3, c.ksplit = ks;
            const double t = predicted_us(M, N, K, c, cus);
            if (t < bar && t < best_t) best = c, best_t = t;
        }
    }
    return best;
}

// Whole rounds first, the remainder as a launch of its own.  A grid of 5.4 rounds of resident
// workgroups ends with a round that runs on a fraction of the CUs.  Cut at a channel where a round
// ends (the resident 128 x 512 tiles cover all token tiles of CUs / token-tiles column tiles), the
// first part runs in whole rounds of the wide tile and the rest is a narrower layer that gets the
// tile shape that suits it.  The gain is small, because the hardware already spreads a partial
// round over the CUs one workgroup each: in the benchmark (graph replay, weights never cached)
// LLaMA-65B gate+up at M = 2048 (5.4 rounds) 576 -> 565 us, LLaMA-7B gate+up (2.7 rounds)
// 161.2 -> 158.8 us.  One round plus a remainder gains nothing and is left alone.
TiledTail tiled_tail(int M, int N, int K)
{
    (void)K;
    TiledTail t{0, 0};
    const int cus = cu_count();
    const int tiles_m = (M + 127) / 128;
    if (M <= 64 || tiles_m > cus || cus % tiles_m != 0) return t;
    const long long per_round = (long long)(cus / tiles_m) * 512;   // output channels one round of 128 x 512 tiles covers
    const long long rounds = N / per_round;
    if (rounds < 2 || N % per_round == 0) return t;
    t.n_first = (int)(rounds * per_round);
    t.nw_first = 8;
    return t;
}

// Tile shape of a plan (tokens x output channels).
static inline void plan_tile(const TiledPlan &p, int &bm, int &bn) { bm = 32 * p.mi, bn = 64 * p.nw; }

size_t tiled_workspace_bytes(int M, int N, int K)
{
    if (tiled_tail(M, N, K).n_first) return 0;   // both launches run without a K split
    const TiledPlan p = tiled_plan(M, N, K);
    if (p.ksplit <= 1) return 0;
    int bm, bn;
    plan_tile(p, bm, bn);
    const size_t tiles = (size_t)((M + bm - 1) / bm) * ((N + bn - 1) / bn);
    return kSplitCounterBytes + tiles * p.ksplit * bm * bn * sizeof(int32_t);
}

template <int G, int NW, int MI, int ST>
static hipError_t launch_tiled_cfg(const LinearArgs &a, int ksplit, void *workspace, hipStream_t st, bool cols = false)
{
    const int tiles_m = (a.M + 32 * MI - 1) / (32 * MI);
    const int tiles_n = (a.N + 64 * NW - 1) / (64 * NW);
    const long long T = (long long)tiles_m * tiles_n * ksplit;
    const long long blocks = ((T + 7) / 8) * 8;
    if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)blocks), block(64 * NW);
    SplitK sk{ksplit, nullptr, nullptr};
    if (ksplit > 1) {
        char *ws = static_cast<char *>(workspace);
        sk.counters = reinterpret_cast<uint32_t *>(ws);
        if ((size_t)tiles_m * tiles_n * sizeof(uint32_t) > kSplitCounterBytes) return hipErrorInvalidValue;   // tiled_plan never splits that many tiles
        sk.partial = reinterpret_cast<int32_t *>(ws + kSplitCounterBytes);
    }
#define DGQ_LAUNCH(KERNEL, ...)                                                                            \
    do {                                                                                                   \
        if (a.acc_out)                                                                                     \
            hipLaunchKernelGGL((KERNEL<G, NW, MI, ST, true>), grid, block, 0, st, a, tiles_m, tiles_n, ##__VA_ARGS__);  \
        else                                                                                               \
            hipLaunchKernelGGL((KERNEL<G, NW, MI, ST, false>), grid, block, 0, st, a, tiles_m, tiles_n, ##__VA_ARGS__); \
    } while (0)
    if (cols) {
        if (ksplit > 1) return hipErrorInvalidValue;
        if (a.zp) DGQ_LAUNCH(linear_tiled_cols_zp_kernel);
        else DGQ_LAUNCH(linear_tiled_cols_kernel);
    } else if (ksplit > 1) {
        if (a.zp) DGQ_LAUNCH(linear_tiled_splitk_zp_kernel, sk);
        else DGQ_LAUNCH(linear_tiled_splitk_kernel, sk);
    } else {
        if (a.zp) DGQ_LAUNCH(linear_tiled_zp_kernel);
        else DGQ_LAUNCH(linear_tiled_kernel);
    }
#undef DGQ_LAUNCH
    return hipGetLastError();
}

template <int G>
static hipError_t launch_tiled_g(const LinearArgs &a, const TiledPlan &p, void *workspace, hipStream_t st, bool cols = false)
{
    if (p.mi == 2) return launch_tiled_cfg<G, 4, 2, 3>(a, p.ksplit, workspace, st, cols);
    if (p.nw == 8) return launch_tiled_cfg<G, 8, 4, 3>(a, p.ksplit, workspace, st, cols);
    return launch_tiled_cfg<G, 4, 4, 3>(a, p.ksplit, workspace, st, cols);
}

// The second of the two launches of a layer cut by tiled_tail: its plan, without a K split.
static TiledPlan tail_plan(int M, int n_rest) { return tiled_base_plan(M, n_rest, cu_count()); }

hipError_t launch_linear_tiled(const LinearArgs &a, void *workspace, hipStream_t st)
{
    const TiledTail t = tiled_tail(a.M, a.N, a.K);
    if (!t.n_first) {
        const TiledPlan p = tiled_plan(a.M, a.N, a.K);
        return a.group == 128 ? launch_tiled_g<128>(a, p, workspace, st) : launch_tiled_g<64>(a, p, workspace, st);
    }
    // first part: channels [0, n_first) in whole rounds
    LinearArgs first = a;
    first.N = t.n_first;
    first.ldo = a.N;
    TiledPlan pf;
    pf.nw = t.nw_first, pf.mi = 4, pf.st = 3, pf.ksplit = 1;
    hipError_t e = a.group == 128 ? launch_tiled_g<128>(first, pf, nullptr, st, true) : launch_tiled_g<64>(first, pf, nullptr, st, true);
    if (e != hipSuccess) return e;
    // the rest: the packed arrays are ordered by blocks of 16 channels, so a range that starts at a
    // multiple of 16 is a contiguous part of each of them
    LinearArgs rest = a;
    const int steps = a.K / 128;
    const int per_word = a.zp ? 2 : 4;   // groups per 32-bit scale word
    const int words = (a.K / a.group + per_word - 1) / per_word;
    rest.N = a.N - t.n_first;
    rest.ldo = a.N;
    rest.qweight = reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(a.qweight) + (size_t)(t.n_first / 16) * steps * 1024);
    rest.scales = reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(a.scales) + (size_t)(t.n_first / 16) * words * 64);
    if (a.s1) rest.s1 = a.s1 + t.n_first;
    if (a.out) rest.out = a.out + t.n_first;
    if (a.acc_out) rest.acc_out = a.acc_out + t.n_first;
    const TiledPlan pr = tail_plan(a.M, rest.N);
    return a.group == 128 ? launch_tiled_g<128>(rest, pr, nullptr, st, true) : launch_tiled_g<64>(rest, pr, nullptr, st, true);
}

void tiled_plan_name(int M, int N, int K, int group, char *buf, size_t buf_bytes)
{
    const TiledTail t = tiled_tail(M, N, K);
    if (!t.n_first) {
        const TiledPlan p = tiled_plan(M, N, K);
        std::snprintf(buf, buf_bytes, "linear_tiled_%skernel<%d, %d, %d, %d, false>", p.ksplit > 1 ? "splitk_" : "", group, p.nw,
                      p.mi, p.st);
        return;
    }
    const TiledPlan pr = tail_plan(M, N - t.n_first);
    std::snprintf(buf, buf_bytes, "linear_tiled_cols_kernel<%d, %d, 4, 3, false> + linear_tiled_cols_kernel<%d, %d, %d, %d, false>",
                  group, t.nw_first, group, pr.nw, pr.mi, pr.st);
}

}  // namespace dgq
