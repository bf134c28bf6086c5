// Decode A8W4 linear for M <= 16 tokens: one 16-token MFMA tile, weights streamed once.
//
// The layer reads K*N/2 bytes of packed weights and almost nothing else, so everything is
// arranged to keep that stream dense and to take the activations off it:
//
//   - One workgroup of 16 wavefronts per CU (a persistent grid).  Wavefront w owns a fixed
//     slice of K (at most SPW steps of 128 k) for the whole kernel and loads its slice of
//     the INT8 activations into registers ONCE; after that the only global loads in the
//     loop are 1 KiB weight chunks (one 128-bit load per lane) and their group scales.
//   - The workgroup walks over 16-column tiles.  For each tile every wavefront expands its
//     chunks in registers (second line of Eq. 2), issues two v_mfma_i32_16x16x64_i8 per
//     chunk (third line of Eq. 2; tokens beyond M repeat the last row and are never stored)
//     and refills each register slot with the same step of the next tile right away, so a
//     wavefront always has SPW KiB of loads in flight.
//   - The 16 partial INT32 tiles are added through LDS (double buffered, one barrier per
//     tile; integer addition is associative, so the split changes no bit).  The first four
//     wavefronts apply sx[m]*s1[n] (first line of Eq. 2) and store fp16.
//   - If K is too long for 16 wavefronts x SPW steps, several workgroups split K: each leaves
//     its INT32 tiles in the workspace and counts itself in; the one that arrives last adds
//     the others' tiles to its own and runs the epilogue (no waiting, no second kernel).
//   - FQ variant: the kernel is handed the fp16 activations and runs the per-token quantizer
//     (Section 3.1, symmetric 8 bits) itself.  A workgroup that is not split over K needs every
//     token's whole row anyway, so while its first weight loads are in flight its 1024 threads
//     share the M*K values out evenly, take the token maxima with LDS atomics, round to INT8
//     and leave the bytes in LDS (in the buffers the column tiles use later), from where every
//     wavefront fetches its slice.  Neither xq nor sx goes through memory and the separate
//     quantizer launch disappears.  Same arithmetic as quant_act_kernel, hence the same bits.
//     Every workgroup repeats the quantizer, so this pays only for small M*K.
#include "dgq_device.hpp"

namespace dgq {
namespace {

constexpr int kWaves = 16;
// A workgroup keeps the finished INT32 tiles of all its column tiles in LDS and stores
// them after the weight loop, so that the loop itself contains no global stores.
constexpr int kMaxTilesPerWg = 32;
// Launch geometry worked out on the host: workgroup wg of K part kpart is block
// (wg << ks_shift) + kpart and walks column tiles wg, wg + cols, ...
struct DecodeGrid {
    int cols;        // workgroups per K part
    int ks_shift;    // log2 of the number of K parts
    int tiles_base;  // every workgroup has this many column tiles ...
    int tiles_rem;   // ... and the first tiles_rem one more
    // K split only: one counter per group of workgroups that share their column tiles (zero
    // before the launch and again after it), and (tiles_base + 1) * 256 INT32 per workgroup
    uint32_t *counters;   // [cols]
    int32_t *partial;     // [cols][parts][(tiles_base + 1) * 256]
};
struct alignas(16) DecodeLds {
    int red[2][kWaves][256];           // partial tiles of the 16 wavefronts, double buffered
    int sums[kMaxTilesPerWg][256];     // finished INT32 tiles
};
static_assert(sizeof(DecodeLds::red) / 2 + sizeof(DecodeLds::sums) == kQuantDecodeStageBytes, "staging area");

// ZP: the scale words hold (S2, ZP) pairs instead of S2 bytes (compile-time).
// FQ: activations arrive as fp16 and are quantized here (needs ksplit == 1, no ACC, no PARTIAL).
// RMS (with FQ): the fp16 input is RMS-normalised and multiplied by gamma first, as
// rmsnorm_quant_act_kernel does it (fp64 up to the rounding to fp32 and then fp16, the squares
// added in the same fixed order).
template <int SPW, int PF, int G, bool ACC, bool PARTIAL, bool ZP, bool FQ, bool RMS = false, bool NT = false>
__device__ __forceinline__ void decode_body(const LinearArgs &a, const DecodeGrid &grid)
{
    // Everything before the first load is one wavefront executing straight-line scalar code at a
    // few cycles per instruction, so it is kept short: no run-time integer divisions (the host
    // passes quotients and remainders), and the K split is a constant 1 where there is none.
    const int ks_shift = PARTIAL ? grid.ks_shift : 0;   // the K split is a power of two
    static_assert(!FQ || (!ACC && !PARTIAL), "the quantizing variant writes fp16 only and sees all of K");
    static_assert(!RMS || FQ, "the normalising variant is a quantizing variant");
    // One block, so that red[1] and sums are contiguous (the FQ variant stages INT8 rows there).
    __shared__ DecodeLds lds;
    int (&red)[2][kWaves][256] = lds.red;
    int (&sums)[kMaxTilesPerWg][256] = lds.sums;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = lane & 15;
    const int kb = lane >> 4;
    const int steps = a.K >> 7;
    const ScaleForm sf = scale_form(ZP ? 1 : 0);  // scale words hold 4 groups (S2 bytes) or 2 (S2, ZP pairs)
    const int gqn = ((a.K / G) + (1 << sf.fsh) - 1) >> sf.fsh;

    // This workgroup's part of K; wavefront w takes steps [p0 + w*SPW, p0 + (w+1)*SPW) of it.
    // Only the last active wavefront can be short; wavefronts past the end only help reduce.
    const int wg_stride = grid.cols;
    const int kpart = (int)blockIdx.x & ((1 << ks_shift) - 1);
    const int wg = (int)blockIdx.x >> ks_shift;
    const int p0 = (steps * kpart) >> ks_shift;
    const int p1 = (steps * (kpart + 1)) >> ks_shift;
    const int active_waves = (p1 - p0 + SPW - 1) / SPW;  // <= kWaves, checked on the host
    const int sb = p0 + wave * SPW;
    const int nst = sb < p1 ? (p1 - sb < SPW ? p1 - sb : SPW) : 0;
    const int my_tiles = grid.tiles_base + (wg < grid.tiles_rem ? 1 : 0);   // tiles wg, wg + cols, ...

    // Epilogue operands, fetched early so that the end of the kernel does not wait on memory, but
    // behind the first weight loads (every wavefront calls this once).  In the epilogue thread x
    // handles element x%256 of tiles x/256, x/256 + 4, ...: a fixed token, and one output
    // channel per tile.
    constexpr int kEarly = 3;
    const int ep_x = threadIdx.x & 255;
    const int ep_m = 4 * ((ep_x & 63) >> 4) + (ep_x >> 6);
    float ep_sx = 0.0f, ep_s1[kEarly] = {0.0f, 0.0f, 0.0f};
    auto load_epilogue_operands = [&]() {
        if (!ACC && ep_m < a.M) {
            if (!FQ) ep_sx = a.sx[ep_m];
#pragma unroll
            for (int k = 0; k < kEarly; ++k) {
                const int ti = (threadIdx.x >> 8) + 4 * k;
                if (ti < my_tiles) ep_s1[k] = a.s1[(wg + ti * wg_stride) * 16 + (ep_x & 15)];
            }
        }
    };

    // FQ (called once by every wavefront, at a point all of them reach): the per-token quantizer
    // run by the whole workgroup, then this wavefront's slice fetched from LDS.
    //   part[16][64]  token maxima per lane slot (fp16 bit patterns), in red[0]: a lane only ever
    //                 updates its own slot, so the LDS atomics of a wavefront do not serialize
    //   tinv, tsx     127/a and a/127 per token, behind part in red[0]
    //   stage         xq[M][K + 16], in red[1] and sums (kQuantDecodeStageBytes).  The 16 bytes
    //                 between rows move each token to the next four LDS banks, so that the 16
    //                 lanes that read the same k of 16 tokens do not collide.
    // Nothing here collides with the column tiles: a wavefront writes red[0] and reads or writes
    // red[1] and sums only behind barriers that come after its last access below.
    constexpr int kVec = FQ ? kQuantDecodeStageBytes / 8 / (kWaves * 64) : 1;   // 8-value vectors per thread
    const int vpr = a.K >> 3;                                                  // vectors per row
    const int nvec = a.M * vpr;
    uint4 v[kVec];
    uint4 gv[RMS ? kVec : 1];
    int tok[kVec];
    if constexpr (FQ) {
        // The fp16 loads go out before the first weight loads, so that waiting for them leaves
        // the weight loads in flight.
        const float inv_vpr = 1.0f / (float)vpr;
        const uint4 *xv = reinterpret_cast<const uint4 *>(a.x16);
#pragma unroll
        for (int i = 0; i < kVec; ++i) {
            const int idx = threadIdx.x + i * (kWaves * 64);
            v[i] = idx < nvec ? xv[idx] : make_uint4(0, 0, 0, 0);
            // idx / vpr without an integer division: (idx + 0.5) / vpr is at least 0.5 / vpr away
            // from an integer, far more than the rounding of this product (idx < 2^13, vpr < 2^13)
            tok[i] = (int)(((float)idx + 0.5f) * inv_vpr);
            if constexpr (RMS)
                gv[i] = idx < nvec ? reinterpret_cast<const uint4 *>(a.gamma)[idx - tok[i] * vpr] : make_uint4(0, 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    auto quantize_rows = [&](uint4 (&xa)[SPW][2]) {
        uint32_t *part = reinterpret_cast<uint32_t *>(&red[0][0][0]);
        float *tinv = reinterpret_cast<float *>(&red[0][4][0]);
        float *tsx = tinv + 16;
        uint8_t *stage = reinterpret_cast<uint8_t *>(&red[1][0][0]);
        if constexpr (RMS) {
            // y = fp16(float(x * r * gamma)), r = 1 / sqrt(mean(x^2) + eps), all in fp64 up to the two
            // roundings.  Every 8-value vector leaves the sum of its squares in an LDS slot of its
            // own (ssq, in the staging area that the quantizer fills later; no atomics), and
            // wavefront w adds up the slots of token w in the one fixed order that
            // rmsnorm_quant_act_kernel uses too (see sum_squares_f64), so both give the same bits.
            double *ssq = reinterpret_cast<double *>(stage);
            double *tr = reinterpret_cast<double *>(&red[0][4][64]);
#pragma unroll
            for (int i = 0; i < kVec; ++i) {
                const int idx = threadIdx.x + i * (kWaves * 64);
                if (idx < nvec) ssq[idx] = sum_squares_f64(v[i]);
            }
            __syncthreads();
            if (wave < a.M) {
                const double *mine = ssq + wave * vpr;
                double total = 0.0;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    double p = 0.0;
                    for (int t = 64 * w + lane; t < vpr; t += 256) p += mine[t];
                    p = wave_sum_f64_lane63(p);
                    total = w == 0 ? p : total + p;
                }
                if (lane == 63) tr[wave] = 1.0 / sqrt(total / (double)a.K + (double)a.eps);
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < kVec; ++i) {
                const int idx = threadIdx.x + i * (kWaves * 64);
                if (idx < nvec) {
                    const double r = tr[tok[i]];
                    const uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
                    const uint32_t gw[4] = {gv[i].x, gv[i].y, gv[i].z, gv[i].w};
                    uint32_t y[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        y[k] = 0;
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            const double xd = (double)half_bits_to_float((w[k] >> (16 * h)) & 0xFFFFu);
                            const double gd = (double)half_bits_to_float((gw[k] >> (16 * h)) & 0xFFFFu);
                            const float p32 = (float)(xd * r * gd);
                            y[k] |= (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)p32) << (16 * h);
                        }
                    }
                    v[i] = make_uint4(y[0], y[1], y[2], y[3]);
                }
            }
        }
        part[threadIdx.x] = 0;                                             // 16 tokens x 64 slots
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kVec; ++i) {
            const int idx = threadIdx.x + i * (kWaves * 64);
            if (idx < nvec) atomicMax(&part[tok[i] * 64 + lane], absmax_bits(v[i], 0));
        }
        __syncthreads();
        {   // wavefront w finishes token w
            const uint32_t mx = wave_max_u32_lane63(part[threadIdx.x]);
            if (lane == 63) {
                const float am = half_bits_to_float(mx);
                tinv[wave] = am != 0.0f ? 127.0f / am : 0.0f;
                tsx[wave] = am != 0.0f ? am / 127.0f : 0.0f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kVec; ++i) {
            const int idx = threadIdx.x + i * (kWaves * 64);
            if (idx < nvec)
                *reinterpret_cast<uint2 *>(stage + tok[i] * (a.K + 16) + (idx - tok[i] * vpr) * 8) =
                    quant_vec_fast(v[i], tinv[tok[i]]);
        }
        ep_sx = tsx[ep_m];
        if (a.sx_out && blockIdx.x == 0 && threadIdx.x < 256 && (ep_x & 15) == 0 && ep_m < a.M)
            a.sx_out[ep_m] = ep_sx;
        __syncthreads();
        if (nst > 0) {
            const int m = j < a.M ? j : a.M - 1;
            const uint4 *sp = reinterpret_cast<const uint4 *>(stage + m * (a.K + 16) + kb * 32);
#pragma unroll
            for (int i = 0; i < SPW; ++i) {
                const int sidx = i < nst ? sb + i : sb;
                xa[i][0] = sp[sidx * 8];
                xa[i][1] = sp[sidx * 8 + 1];
                if (i >= nst) xa[i][0] = xa[i][1] = make_uint4(0, 0, 0, 0);
            }
        }
    };
    uint4 xa[SPW][2];

    if (nst > 0) {
        // activations of this slice: loaded once, kept in registers; slots past the end of
        // a short slice hold zeros, so whatever weights they are multiplied with add nothing
        if constexpr (!FQ) {
            const int m = j < a.M ? j : a.M - 1;
            const uint4 *ap = reinterpret_cast<const uint4 *>(a.xq + (size_t)m * a.K + kb * 32);
#pragma unroll
            for (int i = 0; i < SPW; ++i) {
                const int s = i < nst ? sb + i : sb;
                xa[i][0] = ap[(size_t)s * 8];
                xa[i][1] = ap[(size_t)s * 8 + 1];
            }
            // (slots past the end of a short slice are zeroed after the first weight loads have
            // been issued: anything that touches xa here would wait for these loads first and
            // hold the weight stream back by a memory latency)
            __builtin_amdgcn_sched_barrier(0);
        }

        // per-slot element offsets inside one column tile (a short slice re-reads step sb)
        int qoff[SPW], soff[SPW], ssh[SPW];
#pragma unroll
        for (int i = 0; i < SPW; ++i) {
            const int s = i < nst ? sb + i : sb;
            const int gi = (G == 128) ? s : 2 * s + (kb >> 1);
            qoff[i] = s * 64 + lane;
            soff[i] = (gi >> sf.fsh) * 16 + j;
            ssh[i] = (int)scale_entry_shift(gi, sf);
        }

        uint4 q[PF][SPW];
        uint32_t sw[PF][SPW];
        // NT: the weights of a large layer are read with the streaming (non-temporal) policy: they are
        // used once, and keeping them out of the way of the caches gains 3-9 % where the layer is
        // bound by HBM bandwidth (packed weights of 64 MB and more); smaller layers, which are bound
        // by latency, lose 5-20 % with it and use ordinary loads.
#define DGQ_LOAD_SLOT(P, I, TILE)                                              \
    do {                                                                       \
        const v4i *qp_ = reinterpret_cast<const v4i *>(&a.qweight[(size_t)(TILE) * steps * 64 + qoff[I]]); \
        q[P][I] = __builtin_bit_cast(uint4, NT ? __builtin_nontemporal_load(qp_) : *qp_); \
        sw[P][I] = a.scales[(size_t)(TILE) * gqn * 16 + soff[I]];              \
    } while (0)

        // prologue: PF tiles in flight (tiles past the end re-read the first tile, unused)
        // FQ: a CU cannot take all these requests at once, so a wavefront spends about as long
        // issuing them as the data need to arrive, and the quantizer, which every wavefront must
        // reach, would only start then.  A workgroup with a single column tile has nothing that
        // hides this: there the quantizer runs after the first half of the slots and the rest
        // is requested behind it.  With more tiles the requests all go out first (measured: the
        // early quantizer costs those shapes 0.1-0.3 us, and saves the others 0.2-1.2 us).
        constexpr int kSlotsBeforeQuantizer = (PF * SPW + 1) / 2;
        // (kernels with one tile of requests in flight, the long-K ones, always take the early
        // form, and so do the kernels that normalise first: a second copy of the quantizer would
        // make them spill registers)
        const bool quantize_early = PF == 1 || RMS || my_tiles <= 1;
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int t = p < my_tiles ? wg + p * wg_stride : wg;
#pragma unroll
            for (int i = 0; i < SPW; ++i) {
                DGQ_LOAD_SLOT(p, i, t);
                // issue order = consumption order, so that waiting for the oldest slot
                // leaves all younger loads in flight
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (FQ) {
                    if (p * SPW + i + 1 == kSlotsBeforeQuantizer && quantize_early) {
                        load_epilogue_operands();
                        __builtin_amdgcn_sched_barrier(0);
                        quantize_rows(xa);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        }
        if constexpr (FQ) {
            if (!quantize_early) {
                load_epilogue_operands();
                __builtin_amdgcn_sched_barrier(0);
                quantize_rows(xa);
            }
        } else {
            load_epilogue_operands();
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < SPW; ++i)
                if (i >= nst) xa[i][0] = xa[i][1] = make_uint4(0, 0, 0, 0);
        }

#define DGQ_TILE(P, IT)                                                                              \
    do {                                                                                             \
        const int it_ = (IT);                                                                        \
        const int tn_ = it_ + PF < my_tiles ? wg + (it_ + PF) * wg_stride : wg;                      \
        v4i acc = v4i{0, 0, 0, 0};                                                                   \
        _Pragma("unroll") for (int i = 0; i < SPW; ++i)                                              \
        {                                                                                            \
            const GroupScale gs = group_scale_at(sw[P][i], ssh[i], sf);                              \
            v4i b0, b1;                                                                              \
            expand_cell(q[P][i], gs, b0, b1);                                                        \
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(v4i, xa[i][0]), b0, acc, 0, 0, 0); \
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(v4i, xa[i][1]), b1, acc, 0, 0, 0); \
            DGQ_LOAD_SLOT(P, i, tn_);                                                                \
            __builtin_amdgcn_sched_barrier(0); /* keep each refill right behind its use */           \
        }                                                                                            \
        /* acc[r] of lane l: token 4*(l/16) + r, column tile*16 + l%16 */                            \
        int *mine = &red[it_ & 1][wave][0];                                                          \
        _Pragma("unroll") for (int r = 0; r < 4; ++r) mine[r * 64 + lane] = acc[r];                  \
        __syncthreads();                                                                             \
        if (threadIdx.x < 256) {                                                                     \
            int sum = 0;                                                                             \
            for (int w = 0; w < active_waves; ++w) sum += red[it_ & 1][w][threadIdx.x];              \
            sums[it_][threadIdx.x] = sum;                                                            \
        }                                                                                            \
        /* No second barrier: the next tile writes the other buffer, and that buffer's readers */    \
        /* passed the barrier above only after their reads. */                                       \
    } while (0)

        // Main loop: whole rounds of PF tiles, straight-line, so every wait for a slot leaves
        // the younger PF*SPW - 1 slots in flight.  Then the last my_tiles % PF tiles.
        int it0 = 0;
        for (; it0 + PF <= my_tiles; it0 += PF) {
#pragma unroll
            for (int p = 0; p < PF; ++p) DGQ_TILE(p, it0 + p);
        }
#pragma unroll
        for (int p = 0; p < PF - 1; ++p)
            if (it0 + p < my_tiles) DGQ_TILE(p, it0 + p);
#undef DGQ_TILE
#undef DGQ_LOAD_SLOT
    } else {
        // wavefronts without a slice of K: keep the barrier count and help with the reduction
        load_epilogue_operands();
        if constexpr (FQ) quantize_rows(xa);
        for (int it = 0; it < my_tiles; ++it) {
            __syncthreads();
            if (threadIdx.x < 256) {
                int sum = 0;
                for (int w = 0; w < active_waves; ++w) sum += red[it & 1][w][threadIdx.x];
                sums[it][threadIdx.x] = sum;
            }
        }
    }
    __syncthreads();

    if constexpr (PARTIAL) {
        // K split: this workgroup's tiles go to its block of the workspace, then it counts itself
        // in; the last of the group to arrive adds the other blocks to its tiles and goes on.
        // Stores and loads of partial tiles are relaxed atomics of device scope (they go through to
        // the level of the memory system that all compute units share; no cache is written back
        // or invalidated for them), ordered against the counter by hand: stores complete
        // (vmcnt(0)) before the barrier behind which the workgroup counts itself in, loads are
        // issued after the counter's old value has come back.
        const int parts = 1 << ks_shift;
        const size_t blk_pairs = (size_t)(grid.tiles_base + 1) * 128;
        unsigned long long *mine = reinterpret_cast<unsigned long long *>(grid.partial) + ((size_t)wg * parts + kpart) * blk_pairs;
        unsigned long long *flat = reinterpret_cast<unsigned long long *>(&sums[0][0]);
        for (int x = threadIdx.x; x < my_tiles * 128; x += kWaves * 64)
            __hip_atomic_store(&mine[x], flat[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_s_waitcnt(0x0070);                     // vmcnt(0), lgkmcnt(0): the tiles have reached memory
        __syncthreads();
        uint32_t *arrived = reinterpret_cast<uint32_t *>(&red[0][0][0]);
        if (threadIdx.x == 0)
            *arrived = __hip_atomic_fetch_add(&grid.counters[wg], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (*arrived != (uint32_t)(parts - 1)) return;          // somebody else will finish these tiles
        if (threadIdx.x == 0)                                   // ready for the next launch
            __hip_atomic_store(&grid.counters[wg], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int p = 0; p < parts; ++p) {
            if (p == kpart) continue;
            const unsigned long long *other = reinterpret_cast<const unsigned long long *>(grid.partial) + ((size_t)wg * parts + p) * blk_pairs;
            for (int x = threadIdx.x; x < my_tiles * 128; x += kWaves * 64) {
                const unsigned long long o = __hip_atomic_load(&other[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                int *dst = &sums[0][0] + 2 * x;
                dst[0] += (int)(uint32_t)o;
                dst[1] += (int)(uint32_t)(o >> 32);
            }
        }
        __syncthreads();
    }

    // Epilogue for all tiles of this workgroup.  Element x of a tile: token 4*((x%64)/16) + x/64,
    // column tile*16 + x%16.
    if (ep_m < a.M) {
        int k = 0;
        for (int ti = threadIdx.x >> 8; ti < my_tiles; ti += 4, ++k) {
            const int sum = sums[ti][ep_x];
            const int n = (wg + ti * wg_stride) * 16 + (ep_x & 15);
            if (ACC) {
                a.acc_out[(size_t)ep_m * a.N + n] = sum;
            } else {
                float s1n;
                if (k == 0) s1n = ep_s1[0];
                else if (k == 1) s1n = ep_s1[1];
                else if (k == 2) s1n = ep_s1[2];
                else s1n = a.s1[n];
                const float sc = ep_sx * s1n;
                a.out[(size_t)ep_m * a.N + n] = scaled_sum_to_half_bits(sc, sum);
            }
        }
    }
}

template <int SPW, int PF, int G, bool ACC, bool PARTIAL>
__global__ __launch_bounds__(kWaves * 64) void linear_decode_kernel(LinearArgs a, DecodeGrid grid)
{
    decode_body<SPW, PF, G, ACC, PARTIAL, false, false>(a, grid);
}
template <int SPW, int PF, int G, bool ACC, bool PARTIAL>
__global__ __launch_bounds__(kWaves * 64) void linear_decode_zp_kernel(LinearArgs a, DecodeGrid grid)
{
    decode_body<SPW, PF, G, ACC, PARTIAL, true, false>(a, grid);
}
// the same with streaming loads of the weights (large layers)
template <int SPW, int PF, int G, bool PARTIAL>
__global__ __launch_bounds__(kWaves * 64) void linear_decode_nt_kernel(LinearArgs a, DecodeGrid grid)
{
    decode_body<SPW, PF, G, false, PARTIAL, false, false, false, true>(a, grid);
}
template <int SPW, int PF, int G, bool PARTIAL>
__global__ __launch_bounds__(kWaves * 64) void linear_decode_nt_zp_kernel(LinearArgs a, DecodeGrid grid)
{
    decode_body<SPW, PF, G, false, PARTIAL, true, false, false, true>(a, grid);
}
template <int SPW, int PF, int G>
__global__ __launch_bounds__(kWaves * 64) void quant_linear_decode_nt_kernel(LinearArgs a, DecodeGrid grid)
{
    decode_body<SPW, PF, G, false, false, false, true, false, true>(a, grid);
}
template <int SPW, int PF, int G>
__global__ __launch_bounds__(kWaves * 64) void quant_linear_decode_nt_zp_kernel(LinearArgs a, DecodeGrid grid)
{
    decode_body<SPW, PF, G, false, false, true, true, false, true>(a, grid);
}
// fp16 activations in, quantized by the kernel itself (one workgroup sees the whole of K)
template <int SPW, int PF, int G>
__global__ __launch_bounds__(kWaves * 64) void quant_linear_decode_kernel(LinearArgs a, DecodeGrid grid)
{
    decode_body<SPW, PF, G, false, false, false, true>(a, grid);
}
template <int SPW, int PF, int G>
__global__ __launch_bounds__(kWaves * 64) void quant_linear_decode_zp_kernel(LinearArgs a, DecodeGrid grid)
{
    decode_body<SPW, PF, G, false, false, true, true>(a, grid);
}
// the same with RMSNorm in front of the quantizer
template <int SPW, int PF, int G>
__global__ __launch_bounds__(kWaves * 64) void rmsnorm_quant_linear_decode_kernel(LinearArgs a, DecodeGrid grid)
{
    decode_body<SPW, PF, G, false, false, false, true, true>(a, grid);
}
template <int SPW, int PF, int G>
__global__ __launch_bounds__(kWaves * 64) void rmsnorm_quant_linear_decode_zp_kernel(LinearArgs a, DecodeGrid grid)
{
    decode_body<SPW, PF, G, false, false, true, true, true>(a, grid);
}

// Workgroups per K part for N / 16 column tiles.
int decode_cols(int tiles, int ksplit)
{
    int cols = cu_count() / ksplit;
    if (cols < 1) cols = 1;
    if (cols * kMaxTilesPerWg < tiles) cols = (tiles + kMaxTilesPerWg - 1) / kMaxTilesPerWg;
    if (cols > tiles) cols = tiles;
    return cols;
}

template <int SPW, int PF, int G>
hipError_t launch_spw(const LinearArgs &a, int ksplit, void *workspace, hipStream_t st)
{
    const int tiles = a.N / 16;
    const int cols = decode_cols(tiles, ksplit);
    dim3 grid(cols * ksplit), block(kWaves * 64);
    int ks_shift = 0;
    while ((1 << ks_shift) < ksplit) ++ks_shift;
    if ((1 << ks_shift) != ksplit) return hipErrorInvalidValue;   // decode_plan only makes powers of two
    DecodeGrid dg{cols, ks_shift, tiles / cols, tiles % cols, nullptr, nullptr};
    if (ksplit > 1) {
        char *ws = static_cast<char *>(workspace);
        dg.counters = reinterpret_cast<uint32_t *>(ws);
        if ((size_t)cols * sizeof(uint32_t) > kSplitCounterBytes) return hipErrorInvalidValue;   // cols <= number of CUs
        dg.partial = reinterpret_cast<int32_t *>(ws + kSplitCounterBytes);
    }
    const bool acc = a.acc_out != nullptr;
    const bool nt = decode_streams_weights(a.N, a.K) && !a.gamma;
    if (a.x16) {
        if (ksplit > 1 || acc || (long long)a.M * (a.K + 16) > kQuantDecodeStageBytes) return hipErrorInvalidValue;
        if (a.gamma) {
            if constexpr (SPW > kRmsDecodeMaxStepsPerWave) {
                return hipErrorInvalidValue;
            } else if (a.zp) {
                hipLaunchKernelGGL((rmsnorm_quant_linear_decode_zp_kernel<SPW, PF, G>), grid, block, 0, st, a, dg);
            } else {
                hipLaunchKernelGGL((rmsnorm_quant_linear_decode_kernel<SPW, PF, G>), grid, block, 0, st, a, dg);
            }
        } else if (nt) {
            if (a.zp)
                hipLaunchKernelGGL((quant_linear_decode_nt_zp_kernel<SPW, PF, G>), grid, block, 0, st, a, dg);
            else
                hipLaunchKernelGGL((quant_linear_decode_nt_kernel<SPW, PF, G>), grid, block, 0, st, a, dg);
        } else if (a.zp) {
            hipLaunchKernelGGL((quant_linear_decode_zp_kernel<SPW, PF, G>), grid, block, 0, st, a, dg);
        } else {
            hipLaunchKernelGGL((quant_linear_decode_kernel<SPW, PF, G>), grid, block, 0, st, a, dg);
        }
        return hipGetLastError();
    }
    if (nt && !acc) {
        if (ksplit > 1) {
            if (a.zp)
                hipLaunchKernelGGL((linear_decode_nt_zp_kernel<SPW, PF, G, true>), grid, block, 0, st, a, dg);
            else
                hipLaunchKernelGGL((linear_decode_nt_kernel<SPW, PF, G, true>), grid, block, 0, st, a, dg);
        } else if (a.zp) {
            hipLaunchKernelGGL((linear_decode_nt_zp_kernel<SPW, PF, G, false>), grid, block, 0, st, a, dg);
        } else {
            hipLaunchKernelGGL((linear_decode_nt_kernel<SPW, PF, G, false>), grid, block, 0, st, a, dg);
        }
        return hipGetLastError();
    }
    if (ksplit > 1) {
        if (a.zp) {
            if (acc)
                hipLaunchKernelGGL((linear_decode_zp_kernel<SPW, PF, G, true, true>), grid, block, 0, st, a, dg);
            else
                hipLaunchKernelGGL((linear_decode_zp_kernel<SPW, PF, G, false, true>), grid, block, 0, st, a, dg);
        } else if (acc) {
            hipLaunchKernelGGL((linear_decode_kernel<SPW, PF, G, true, true>), grid, block, 0, st, a, dg);
        } else {
            hipLaunchKernelGGL((linear_decode_kernel<SPW, PF, G, false, true>), grid, block, 0, st, a, dg);
        }
    } else if (a.zp) {
        if (acc)
            hipLaunchKernelGGL((linear_decode_zp_kernel<SPW, PF, G, true, false>), grid, block, 0, st, a, dg);
        else
            hipLaunchKernelGGL((linear_decode_zp_kernel<SPW, PF, G, false, false>), grid, block, 0, st, a, dg);
    } else if (acc) {
        hipLaunchKernelGGL((linear_decode_kernel<SPW, PF, G, true, false>), grid, block, 0, st, a, dg);
    } else {
        hipLaunchKernelGGL((linear_decode_kernel<SPW, PF, G, false, false>), grid, block, 0, st, a, dg);
    }
    return hipGetLastError();
}

template <int G>
hipError_t launch_g(const LinearArgs &a, const DecodePlan &p, void *workspace, hipStream_t st)
{
    switch (p.spw) {
    case 1: return launch_spw<1, 4, G>(a, p.ksplit, workspace, st);
    case 2: return launch_spw<2, 2, G>(a, p.ksplit, workspace, st);
    case 3: return launch_spw<3, 2, G>(a, p.ksplit, workspace, st);
    case 4: return launch_spw<4, 1, G>(a, p.ksplit, workspace, st);
    case 5: return launch_spw<5, 1, G>(a, p.ksplit, workspace, st);
    case 6: return launch_spw<6, 1, G>(a, p.ksplit, workspace, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

// Compute units of the current device (256 if there is none: host-only queries).
int cu_count()
{
    static int n = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
            v = 256;
        return v;
    }();
    return n;
}

// Layers whose packed weights reach 64 MB are read with streaming loads (see DGQ_LOAD_SLOT).
bool decode_streams_weights(int N, int K) { return (long long)N * K / 2 >= (64LL << 20); }

DecodePlan decode_plan(int K)
{
    const int steps = K / 128;
    DecodePlan p;
    p.ksplit = 1;
    while (((steps + p.ksplit - 1) / p.ksplit + kWaves - 1) / kWaves > kDecodeMaxStepsPerWave) p.ksplit *= 2;
    p.spw = ((steps + p.ksplit - 1) / p.ksplit + kWaves - 1) / kWaves;
    // spw steps per wavefront x pf tiles ahead = KiB of weight loads in flight per wavefront
    p.pf = p.spw <= 1 ? 4 : (p.spw <= 3 ? 2 : 1);
    return p;
}

size_t decode_workspace_bytes(int M, int N, int K)
{
    (void)M;   // the partial tiles always hold 16 tokens
    const int ks = decode_plan(K).ksplit;
    if (ks <= 1) return 0;
    const int tiles = N / 16;
    const int cols = decode_cols(tiles, ks);
    return kSplitCounterBytes + (size_t)cols * ks * (tiles / cols + 1) * 256 * sizeof(int32_t);
}

hipError_t launch_linear_decode(const LinearArgs &a, void *workspace, hipStream_t st)
{
    if (a.M > kDecodeMaxM) return hipErrorInvalidValue;
    const DecodePlan p = decode_plan(a.K);
    return a.group == 128 ? launch_g<128>(a, p, workspace, st) : launch_g<64>(a, p, workspace, st);
}

}  // namespace dgq
