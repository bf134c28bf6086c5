// Internal declarations shared by the HIP translation units of libdgq.so.
// Not part of the public ABI (that is include/dgq.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "dgq.h"

namespace dgq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned short v2u16 __attribute__((ext_vector_type(2)));

// ---- INT4 -> INT8 expansion in registers (second line of Eq. 2) -------------------
//
// A 32-bit word holds eight stored nibbles u.  The even nibbles (low halves of the four
// bytes) and the odd nibbles (high halves) are separated into two words of four bytes each;
// every byte is then turned into the signed INT8 value s2 * (u - zp):
//
//   r = s2*u + (128 - zp*s2) is the wanted value plus 128, so it lies in [0, 255] whenever
//   the value fits INT8 (which packing has checked).  One packed 16-bit multiply-add over
//   byte pairs computes (r0 + 256*r1) modulo 2^16: intermediate products may wrap, the sum
//   cannot, because both r are bytes.  Flipping bit 7 of each byte then subtracts the 128
//   again in two's complement.  With the constant zero point 8 of the signed-nibble format
//   and s2 <= 15, r lies in [8, 233].
struct GroupScale {
    uint32_t mul;  // s2 in both 16-bit halves
    uint32_t add;  // (128 - zp*s2) modulo 256 in all four bytes
};

__device__ __forceinline__ GroupScale make_group_scale(uint32_t s2, uint32_t zp)
{
    GroupScale g;
    g.mul = s2 | (s2 << 16);
    // 0x8080 - s2*zp*0x0101 per 16-bit half (mod 2^16): -0x0101 = 0xFEFF
    const uint32_t z2 = zp | (zp << 16);
    const v2u16 f = __builtin_bit_cast(v2u16, z2) * (v2u16){0xFEFF, 0xFEFF};
    const v2u16 r = __builtin_bit_cast(v2u16, g.mul) * f + (v2u16){0x8080, 0x8080};
    g.add = __builtin_bit_cast(uint32_t, r);
    return g;
}

// The scale array has one of two forms (LinearArgs::zp): 0 = one byte per group and column,
// the group scale S2, with the constant zero point 8; 1 = two bytes, S2 then the zero point.
// A 32-bit word therefore holds 4 or 2 consecutive groups of one column.
// Everything that depends on the form is a handful of uniform constants, so that the kernels'
// loops contain no branch on it.
struct ScaleForm {
    int fsh;         // log2 of the groups per word: word index of group gi is gi >> fsh
    uint32_t gmask;  // groups per word - 1
    uint32_t width;  // bits per group
    uint32_t zmask;  // 0xFF if the entry carries a zero point, else 0
    uint32_t zor;    // the constant zero point 8 if it does not
};
__device__ __forceinline__ ScaleForm scale_form(int zp_form)
{
    ScaleForm f;
    f.fsh = zp_form ? 1 : 2;
    f.gmask = zp_form ? 1u : 3u;
    f.width = zp_form ? 16u : 8u;
    f.zmask = zp_form ? 0xFFu : 0u;
    f.zor = zp_form ? 0u : 8u;
    return f;
}
__device__ __forceinline__ uint32_t scale_entry_shift(int gi, const ScaleForm &f) { return ((uint32_t)gi & f.gmask) * f.width; }
__device__ __forceinline__ GroupScale group_scale_at(uint32_t word, uint32_t shift, const ScaleForm &f)
{
    const uint32_t e = word >> shift;
    return make_group_scale(e & 0xFFu, ((e >> 8) & f.zmask) | f.zor);
}

__device__ __forceinline__ uint32_t scale_bytes(uint32_t four_nibbles_in_bytes, const GroupScale &g)
{
    v2u16 a = __builtin_bit_cast(v2u16, four_nibbles_in_bytes);
    v2u16 m = __builtin_bit_cast(v2u16, g.mul);
    v2u16 c = __builtin_bit_cast(v2u16, g.add);
    v2u16 r = a * m + c;
    return __builtin_bit_cast(uint32_t, r) ^ 0x80808080u;
}

// One 16-byte cell (32 nibbles of one column, 32 consecutive k) -> two MFMA operands:
// `first` = W_s8 of the cell's k 0..15 (low nibbles), `second` = k 16..31 (high nibbles).
__device__ __forceinline__ void expand_cell(const uint4 &q, const GroupScale &g, v4i &first, v4i &second)
{
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        first[v] = (int)scale_bytes(w[v] & 0x0F0F0F0Fu, g);
        second[v] = (int)scale_bytes((w[v] >> 4) & 0x0F0F0F0Fu, g);
    }
}

// Epilogue of Eq. 2 for one element: the fp32 product scale * float(acc), then ONE more rounding to
// fp16.  The two roundings are kept apart on purpose: fused into a mixed-precision multiply that
// rounds the exact product straight to fp16, the result differs from the stated definition in
// the rare cases where the fp32 rounding crosses an fp16 tie.
__device__ __forceinline__ unsigned short scaled_sum_to_half_bits(float scale, int acc)
{
    float p = scale * (float)acc;
    asm("" : "+v"(p));   // opaque to the optimizer, free to be scheduled
    return __builtin_bit_cast(unsigned short, (_Float16)p);
}

// ---- per-token activation quantizer arithmetic (Section 3.1, symmetric, 8 bits) -------
// Shared by the stand-alone quantizer kernels and by the decode kernel that quantizes its own
// activations, so that both produce the same bytes: the absolute maximum a of a token is taken
// on fp16 bit patterns (integer order = numeric order for non-negative values), the caller forms
// sx = a / 127 and inv = 127 / a (one IEEE division each), and every element becomes
// clamp(rint(float(x) * inv), -127, 127).
__device__ __forceinline__ uint32_t absmax_bits(const uint4 &v, uint32_t m)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint32_t lo = w[i] & 0x7FFFu, hi = (w[i] >> 16) & 0x7FFFu;
        m = lo > m ? lo : m;
        m = hi > m ? hi : m;
    }
    return m;
}

__device__ __forceinline__ float half_bits_to_float(uint32_t h)
{
    return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
}

__device__ __forceinline__ uint32_t quant_one(uint32_t hbits, float inv)
{
    float q = rintf(half_bits_to_float(hbits) * inv);
    q = fminf(fmaxf(q, -127.0f), 127.0f);
    return (uint32_t)((int)q) & 0xFFu;
}

__device__ __forceinline__ uint2 quant_vec(const uint4 &v, float inv)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t b[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        b[2 * i] = quant_one(w[i] & 0xFFFFu, inv);
        b[2 * i + 1] = quant_one(w[i] >> 16, inv);
    }
    uint2 r;
    r.x = b[0] | (b[1] << 8) | (b[2] << 16) | (b[3] << 24);
    r.y = b[4] | (b[5] << 8) | (b[6] << 16) | (b[7] << 24);
    return r;
}

// The same bytes as quant_vec for finite inputs, in about a quarter of the instructions, for
// the decode kernel in which every workgroup quantizes all tokens again.  |x * inv| never
// exceeds 127 * (1 + 2^-23) because |x| <= a and inv = fl(127 / a), so the clamp is idle; adding
// 1.5 * 2^23 to the fp32 product rounds it to the nearest integer, ties to even, exactly as
// rintf does, and leaves that integer's two's complement in the low mantissa bits.
__device__ __forceinline__ uint32_t quant_bits_fast(uint32_t hbits, float inv)
{
    const float t = half_bits_to_float(hbits) * inv;
    const float r = t + 12582912.0f;
    return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ uint2 quant_vec_fast(const uint4 &v, float inv)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t b[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        b[2 * i] = quant_bits_fast(w[i] & 0xFFFFu, inv);
        b[2 * i + 1] = quant_bits_fast(w[i] >> 16, inv);
    }
    uint2 r;
    r.x = (b[0] & 0xFFu) | ((b[1] & 0xFFu) << 8) | ((b[2] & 0xFFu) << 16) | (b[3] << 24);
    r.y = (b[4] & 0xFFu) | ((b[5] & 0xFFu) << 8) | ((b[6] & 0xFFu) << 16) | (b[7] << 24);
    return r;
}

// Maximum of an unsigned value over the 64 lanes of a wavefront with data-parallel-primitive
// moves (no LDS round trips): within quads, within rows of 16, then row to row.  LANE 63 holds
// the result; a lane whose source is masked off receives 0, the identity of the maximum.
__device__ __forceinline__ uint32_t wave_max_u32_lane63(uint32_t mx)
{
#define DGQ_DPP_MAX(CTRL, ROWS)                                                                          \
    do {                                                                                                 \
        const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mx, (CTRL), (ROWS), 0xF, false); \
        mx = o > mx ? o : mx;                                                                            \
    } while (0)
    DGQ_DPP_MAX(0xB1, 0xF);    // quad_perm [1,0,3,2]
    DGQ_DPP_MAX(0x4E, 0xF);    // quad_perm [2,3,0,1]
    DGQ_DPP_MAX(0x124, 0xF);   // row_ror 4
    DGQ_DPP_MAX(0x128, 0xF);   // row_ror 8
    DGQ_DPP_MAX(0x142, 0xA);   // row_bcast 15 into rows 1 and 3
    DGQ_DPP_MAX(0x143, 0xC);   // row_bcast 31 into rows 2 and 3
#undef DGQ_DPP_MAX
    return mx;
}

// ---- sum of squares of a token for RMSNorm, in ONE fixed order for every kernel -------------
// Both kernels that normalise (the stand-alone producer and the decode kernel that normalises
// and quantizes its own activations) add the squares of a row of K = 8 * nvec values like this,
// all in fp64, so that they derive the same factor bit for bit:
//   1. s_v      = the eight squares of 8-value vector v, added in element order starting from 0
//   2. P[w][l]  = s_v for v = 64*w + l, 64*w + l + 256, ... (increasing v, starting from 0),
//                 w = 0..3, l = 0..63
//   3. W[w]     = the sum of P[w][0..63] by the lane-exchange tree of wave_sum_f64_lane63
//   4. total    = ((W[0] + W[1]) + W[2]) + W[3]
__device__ __forceinline__ double sum_squares_f64(const uint4 &v)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    double ss = 0.0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const double lo = (double)half_bits_to_float(w[k] & 0xFFFFu), hi = (double)half_bits_to_float(w[k] >> 16);
        ss += lo * lo;
        ss += hi * hi;
    }
    return ss;
}
// Sum over the 64 lanes with data-parallel-primitive moves of both halves of the double (same
// lane pattern as wave_max_u32_lane63; a masked-off source contributes +0.0).  LANE 63 holds
// the result.
__device__ __forceinline__ double wave_sum_f64_lane63(double ss)
{
#define DGQ_DPP_ADD(CTRL, ROWS)                                                                            \
    do {                                                                                                   \
        const uint2 b_ = __builtin_bit_cast(uint2, ss);                                                    \
        uint2 o_;                                                                                          \
        o_.x = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)b_.x, (CTRL), (ROWS), 0xF, false);            \
        o_.y = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)b_.y, (CTRL), (ROWS), 0xF, false);            \
        ss += __builtin_bit_cast(double, o_);                                                              \
    } while (0)
    DGQ_DPP_ADD(0xB1, 0xF);    // quad_perm [1,0,3,2]
    DGQ_DPP_ADD(0x4E, 0xF);    // quad_perm [2,3,0,1]
    DGQ_DPP_ADD(0x124, 0xF);   // row_ror 4
    DGQ_DPP_ADD(0x128, 0xF);   // row_ror 8
    DGQ_DPP_ADD(0x142, 0xA);   // row_bcast 15 into rows 1 and 3
    DGQ_DPP_ADD(0x143, 0xC);   // row_bcast 31 into rows 2 and 3
#undef DGQ_DPP_ADD
    return ss;
}

// ---- kernel launchers (defined one per .hip file) ----------------------------------
hipError_t launch_quant_act(const uint16_t *x, int M, int K, int8_t *xq, float *sx, hipStream_t st);
hipError_t launch_rmsnorm_quant_act(const uint16_t *x, const uint16_t *gamma, int M, int K, float eps, int8_t *xq,
                                    float *sx, hipStream_t st);
hipError_t launch_silu_mul_quant_act(const uint16_t *GU, int M, int I, int8_t *xq, float *sx, hipStream_t st);
hipError_t launch_quant_act_static(const uint16_t *x, int M, int K, float s, int8_t *xq, float *sx, hipStream_t st);
hipError_t launch_smooth_scales(const uint16_t *X, int M, int K, int r, float *k, float *z, hipStream_t st);
hipError_t launch_smooth_apply(const uint16_t *W, const uint16_t *X, const float *k, int M, int K, int N,
                               uint16_t *Wout, uint16_t *Xout, hipStream_t st);
hipError_t launch_quantize_rtn(const uint16_t *W, int K, int N, int group, int8_t *w4, uint8_t *s2,
                               float *s1, hipStream_t st);
hipError_t launch_quantize_grid(const uint16_t *W, int K, int N, int group, int n_alpha, float step, uint8_t *u4,
                                uint8_t *zp, uint8_t *s2, float *s1, float *sprime, hipStream_t st);
size_t quantize_grid_act_workspace_bytes(int M, int K, int N, int group);
hipError_t launch_quantize_grid_act(const uint16_t *W, const uint16_t *X, const int8_t *xq, const float *sx, int M, int K,
                                    int N, int group, int n_alpha, float step, uint8_t *u4, uint8_t *zp, uint8_t *s2,
                                    float *s1, float *workspace, hipStream_t st);
hipError_t launch_pack(const int8_t *w4, const uint8_t *s2, int K, int N, int group, void *qweight,
                       void *scales, int32_t *bad_count, hipStream_t st);
hipError_t launch_unpack(const void *qweight, const void *scales, int zp_form, int K, int N, int group,
                         int8_t *w_s8, hipStream_t st);
hipError_t launch_pack_zp(const uint8_t *u4, const uint8_t *s2, const uint8_t *zp, int K, int N, int group,
                          void *qweight, void *scales_zp, int32_t *bad_count, hipStream_t st);

struct LinearArgs {
    const int8_t *xq;
    const float *sx;       // null in acc mode
    const uint4 *qweight;
    const uint32_t *scales;
    const float *s1;       // null in acc mode
    uint16_t *out;         // fp16 bits, null in acc mode
    int32_t *acc_out;      // null in fp16 mode
    int M, N, K, group;
    int zp;                // form of `scales`: 0 = S2 bytes (zero point 8), 1 = (S2, ZP) byte pairs
    // Only for the decode kernel that quantizes its own activations (then xq and sx are null):
    const uint16_t *x16;   // fp16 bits [M][K]
    float *sx_out;         // optional: the token scales it derived, [M]
    const uint16_t *gamma; // optional, fp16 bits [K]: RMS-normalise x and multiply by gamma first
    float eps;             // added to the mean square
    // Only for the tiled kernels that compute a range of output channels of a wider layer (the
    // pointers above then start at the range's first channel, N is its width): elements between the
    // starts of two token rows of out / acc_out.
    int ldo;
};
// A workspace that a K split uses starts with this many bytes of arrival counters (one 32-bit
// word per tile or workgroup column, at most kSplitCounterBytes / 4 of them), whatever the shape
// and the entry point: they are zero before a launch and zero again after it, so a buffer that
// was cleared once serves any sequence of calls.  The partial sums follow.
constexpr size_t kSplitCounterBytes = 65536;
// Largest M the weight-streaming kernels take.
constexpr int kStreamMaxM = 64;
// Decode kernel (one 16-token tile, activations resident in registers).
constexpr int kDecodeMaxM = 16;
constexpr int kDecodeMaxStepsPerWave = 6;  // 8 would spill at 128 VGPRs
// The variant that quantizes its own activations stages xq[M][K] in LDS that the column tiles
// use afterwards (48 KiB), and every workgroup repeats the quantizer: only for small M * K.
constexpr int kQuantDecodeStageBytes = 49152;
// With RMSNorm in front the kernel also holds a gamma vector per activation vector: up to four
// steps per wavefront (K <= 8192, the hidden sizes that feed a block's first linears).
constexpr int kRmsDecodeMaxStepsPerWave = 4;
int cu_count();   // compute units of the current device; 256 when there is no device
struct DecodePlan {
    int spw;     // steps of 128 k per wavefront (template SPW)
    int pf;      // column tiles prefetched ahead (template PF)
    int ksplit;  // workgroups sharing one column tile's K
};
DecodePlan decode_plan(int K);
bool decode_streams_weights(int N, int K);   // large layer: the decode kernel reads its weights with streaming loads
size_t decode_workspace_bytes(int M, int N, int K);
struct StreamPlan {
    int mtiles;  // 16-token tiles (template MT)
    int waves;   // wavefronts per workgroup = K split (template W)
    int depth;   // steps of loads in flight (template D)
};
StreamPlan stream_plan(int M, int N, int K);
hipError_t launch_linear_decode(const LinearArgs &a, void *workspace, hipStream_t st);
hipError_t launch_linear_stream(const LinearArgs &a, hipStream_t st);
struct TiledPlan {
    int nw;      // wavefronts per workgroup, 64 output channels each (template NW)
    int mi;      // 32-token blocks per tile (template MI)
    int st;      // stages of operands in flight or in use (template ST)
    int ksplit;  // workgroups that share one tile, each taking a part of K
};
TiledPlan tiled_plan(int M, int N, int K);
// A layer whose tiles fill the CUs in two or more whole rounds plus a remainder is run as two
// launches: the first n_first output channels (whole rounds of 128 x 512 tiles when nw_first is 8,
// of 128 x 256 tiles when it is 4) and the rest as a problem of its own.  n_first = 0: one launch.
struct TiledTail {
    int n_first;
    int nw_first;
};
TiledTail tiled_tail(int M, int N, int K);
// Name of the kernel(s) launch_linear_tiled would launch, as a profiler shows them (without the namespace).
void tiled_plan_name(int M, int N, int K, int group, char *buf, size_t buf_bytes);
size_t tiled_workspace_bytes(int M, int N, int K);
hipError_t launch_linear_tiled(const LinearArgs &a, void *workspace, hipStream_t st);

hipError_t launch_bmm_s8(const int8_t *A, const int8_t *B, const float *sa, const float *sb, uint16_t *out, int32_t *acc_out,
                         int batch, int M, int N, int K, hipStream_t st);

hipError_t launch_probe_read(const void *src, size_t bytes, uint32_t *sink, int workgroups, hipStream_t st);
hipError_t launch_probe_mfma(const void *operands, size_t bytes, int iters, uint32_t *sink, int workgroups, hipStream_t st);

}  // namespace dgq
