/*
 * dgq.h - C ABI of the MI355X (gfx950) Dual Grained Quantization A8W4 linear layer.
 *
 * The layer is Eq. 2 of the DGQ paper (arXiv 2310.04836, Section 3.2):
 *
 *     s     = s_X * s1                       per-token x per-output-channel scale
 *     W_s8  = S2 * (W_u4 - ZP)               INT4 -> INT8, group-wise integer scale
 *     O_f16 = s * (X_s8 W_s8)                one INT8 GEMM over all of K, INT32 sums
 *
 * with a constant zero point ZP = 8 (signed nibbles w4 = W_u4 - 8 in [-8, 7]) and
 * integer group scales S2 in [1, 15].
 *
 * Orientation (the paper's): X is [M][K] (tokens x input channels), W is [K][N]
 * (input x output channels, N contiguous), groups are `group` consecutive k.
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers unless a parameter says "host".
 *   - The caller owns every buffer; the library allocates nothing, returns no handles
 *     and keeps no state that a call can change (the test hooks take the kernel path as
 *     an argument).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream) and the call returns without synchronising.
 *   - Dense row-major tensors, no strides.  Device pointers must be 16-byte aligned.
 *   - Shape rules: M >= 1, K % 128 == 0, 128 <= K <= 131072 (INT32 sums cannot wrap),
 *     N % 16 == 0, group in {64, 128}.
 *   - Argument errors (every status but DGQ_ERR_HIP) are found on the host and returned
 *     BEFORE anything is launched.  DGQ_ERR_HIP reports a failed launch; where a call
 *     enqueues two kernels (a quantizer in front of the linear; a wide layer run as whole
 *     rounds of tiles plus a remainder) the first may already be enqueued when the second fails.
 *   - NaN/Inf activations give unspecified outputs, not an error.
 *   - Thread-safe; calls on the same buffers must be ordered by the caller.
 */
#ifndef DGQ_H
#define DGQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DGQ_API __attribute__((visibility("default")))

typedef int dgq_status;
enum {
    DGQ_OK = 0,
    DGQ_ERR_NULL = -1,      /* a required pointer is NULL                                  */
    DGQ_ERR_SHAPE = -2,     /* M, N, K or group breaks a shape rule                        */
    DGQ_ERR_ALIGN = -3,     /* a device pointer is not 16-byte aligned                     */
    DGQ_ERR_RANGE = -4,     /* a scalar argument (eps, scale, pct, alpha grid, path) is out of range */
    DGQ_ERR_WORKSPACE = -5, /* workspace_bytes is smaller than dgq_linear_workspace_bytes  */
    DGQ_ERR_HIP = -6        /* a HIP call failed; see dgq_last_hip_error()                 */
};

/* Version of the packed weight format written by dgq_pack_weights (see below). */
#define DGQ_LAYOUT_VERSION 1

/* Static, NUL-terminated description of a status code (host). */
DGQ_API const char *dgq_status_string(dgq_status st);

/* hipError_t (as int) of the most recent DGQ_ERR_HIP on the calling thread; 0 if none. */
DGQ_API int dgq_last_hip_error(void);

/* Returns DGQ_LAYOUT_VERSION of the loaded library. */
DGQ_API int dgq_layout_version(void);

/*
 * Sizes of the packed operands of Eq. 2 for a [K][N] weight (host function, nothing
 * launched): qweight_bytes = K*N/2 (two nibbles per byte),
 * scales_bytes = (N/16) * ceil((K/group)/4) * 64 (one byte per group and column,
 * groups padded to a multiple of four).
 */
DGQ_API dgq_status dgq_packed_sizes(int K, int N, int group, size_t *qweight_bytes, size_t *scales_bytes);

/*
 * Scratch needed by dgq_linear_a8w4 for this problem (host function).  May be 0, in which
 * case `workspace` may be NULL.  Non-zero where several workgroups split the K of a tile:
 * M <= 16 with very long K, and larger M for shapes with few tiles.  It then holds 64 KiB of
 * arrival counters (one per tile) followed by the INT32 partial sums of every part (about
 * parts * M * N * 4 bytes, M and N rounded up to whole tiles, parts <= 8).
 *
 * WORKSPACE CONTRACT (every call that takes a workspace): the buffer must be ZERO-FILLED
 * once before its first use (hipMemset after allocating it).  The counters always sit in the
 * first 64 KiB, whatever the shape and the entry point, and a call leaves them zero again, so
 * the same buffer serves any sequence of calls it is large enough for without being cleared
 * in between; the rest of its contents is undefined before and after.  Two calls that may overlap in time must not share a workspace.  (A call that is
 * torn down while its kernels run, e.g. by a device reset, may leave counters behind: clear
 * the buffer again.)
 *
 * dgq_linear_acc_workspace_bytes is the same for the test hooks dgq_linear_a8w4_acc /
 * _zp_acc, which can force a kernel path (see there).
 */
DGQ_API dgq_status dgq_linear_workspace_bytes(int M, int N, int K, int group, size_t *bytes);
DGQ_API dgq_status dgq_linear_acc_workspace_bytes(int M, int N, int K, int group, int path, size_t *bytes);

/*
 * Offline packing of the integer operands of Eq. 2 (W_u4 - ZP and S2) into the
 * device format.
 *   w4       in  [K][N] int8, signed nibble values in [-8, 7]
 *   s2       in  [K/group][N] uint8, group scales in [1, 15]
 *   qweight  out dgq_packed_sizes().qweight_bytes
 *   scales   out dgq_packed_sizes().scales_bytes
 *   bad_count in/out, nullable: one int32 the caller has zeroed; the kernel adds the
 *            number of inputs outside the ranges above (such a nibble is packed as 0,
 *            such a scale as 1).  Inside the ranges |S2 * w4| <= 120, so the paper's
 *            constraint W_s8 in [-128, 127] (beside Eq. 4) holds for every packed weight.
 * The channel scale s1 of Eq. 2 is not an argument: it is used only by the epilogue, as a
 * plain [N] float array that needs no packing, and goes straight to dgq_linear_a8w4.
 *
 * Format, version 1.  Stored nibble u = w4 + 8.  qweight is a sequence of 16-byte cells;
 * element (k, n) is in cell ((n/16)*(K/128) + k/128)*64 + ((k%128)/32)*16 + n%16, byte
 * k%16 of the cell, low nibble if k%32 < 16, else high nibble.  The scale of group gi
 * and column n is byte ((n/16)*ceil(ng/4) + gi/4)*64 + (n%16)*4 + gi%4 of scales;
 * padding bytes are 0.  One 128-bit load per lane therefore feeds two INT8 MFMA
 * operands (16 consecutive k each) of one column.
 */
DGQ_API dgq_status dgq_pack_weights(const int8_t *w4, const uint8_t *s2, int K, int N, int group,
                            void *qweight, void *scales, int32_t *bad_count, void *stream);

/*
 * Test hook: expands packed weights back to W_s8[K][N] = S2 * (W_u4 - 8) (second line
 * of Eq. 2), the tensor that otherwise only exists in registers.
 */
DGQ_API dgq_status dgq_unpack_weights(const void *qweight, const void *scales, int K, int N, int group,
                              int8_t *w_s8, void *stream);

/*
 * Round-to-nearest dual-grained weight quantizer (the "RTN" scheme of Table 1; symmetric
 * scale of Section 3.1; S = s1 * S2 of Eq. 5), used to turn synthetic fp16 weights into
 * the integer operands:
 *   S'[j][n] = max_{k in group j}|W[k][n]| / 7,  s1[n] = max_j S'[j][n] / 15,
 *   s2[j][n] = clamp(round(S'/s1), 1, 15),  w4 = clamp(round(W / (s1*s2)), -8, 7),
 * fp32 arithmetic, IEEE division, ties to even; a zero column gives s1=1, s2=1, w4=0.
 *   W   in  [K][N] fp16 (raw bits as uint16_t)
 *   w4  out [K][N] int8;  s2 out [K/group][N] uint8;  s1 out [N] float
 */
DGQ_API dgq_status dgq_quantize_weights_rtn(const uint16_t *W, int K, int N, int group,
                                    int8_t *w4, uint8_t *s2, float *s1, void *stream);

/*
 * Per-token dynamic symmetric INT8 activation quantizer (Section 3.1 symmetric case,
 * "per-token dynamic activation quantization" of Section 4.1):
 *   a = max_k |x[m][k]|,  sx[m] = a/127,  xq = clamp(round(x * (127/a)), -127, 127),
 * fp32, ties to even; a zero row gives sx = 0, xq = 0.
 *   x   in  [M][K] fp16 (raw bits);  xq out [M][K] int8;  sx out [M] float
 */
DGQ_API dgq_status dgq_quant_act(const uint16_t *x, int M, int K, int8_t *xq, float *sx, void *stream);

/*
 * Percentile clipping smoothing (Section 3.4, Eq. 6), offline.  From calibration activations
 *   z_j = max_m |X[m][j]|,  t = the r-th largest z with r = ceil(pct * K) (nearest rank),
 *   k_j = max(z_j / t, 1)                                (all ones if t is 0)
 * so fewer than r outlier channels get a scale above 1 (the paper uses pct = 0.005).
 *   X   in  [M][K] fp16 (raw bits), M <= 65535;  k out [K] float
 *   workspace  at least K*4 bytes (the channel maxima)
 * Errors: DGQ_ERR_RANGE unless 0 < pct <= 1.
 */
DGQ_API dgq_status dgq_smooth_scales(const uint16_t *X, int M, int K, float pct, float *k,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * Moves the smoothing scale from the activations into the weights (Section 3.4):
 *   Wout[j][n] = fp16(k_j * W[j][n])   if W is not NULL ([K][N] fp16)
 *   Xout[m][j] = fp16(X[m][j] / k_j)   if X is not NULL ([M][K] fp16)
 * fp32 arithmetic, one rounding to fp16; K <= 131072.  In a model the division is folded into the
 * producer of X; the entry point exists so that the identity (X/k)(kW) = XW can be exercised.
 */
DGQ_API dgq_status dgq_smooth_apply(const uint16_t *W, const uint16_t *X, const float *k, int M, int K, int N,
                            uint16_t *Wout, uint16_t *Xout, void *stream);

/*
 * The activation quantizer folded into its producer, for the second linear layer of a gated
 * MLP (the per-token statistics pass that Section 4.2 names as a cost of dynamic quantization
 * then needs no kernel and no round trip of its own):
 *   h[m][i] = fp16( float( silu(g) * u ) ),  g = gate_up[m][i],  u = gate_up[m][I + i],
 *   silu(g) = g / (1 + exp(-g))  evaluated with the product in fp64,
 * then xq, sx = dgq_quant_act(h).  h is never written.
 *   gate_up in [M][2*I] fp16 (raw bits): the output of the fused gate+up linear, gate columns first
 *   xq out [M][I] int8;  sx out [M] float;   I % 128 == 0, 128 <= I <= 24576
 *
 * dgq_rmsnorm_quant_act does the same for the producer of a block's first linears (qkv, gate+up):
 *   y[m][k] = fp16( float( x * (1 / sqrt(mean_k x^2 + eps)) * gamma[k] ) )   evaluated in fp64,
 *   then xq, sx = dgq_quant_act(y).   x in [M][K] fp16, gamma in [K] fp16, 0 <= eps < 1
 *   (DGQ_ERR_RANGE otherwise), K % 128 == 0, 128 <= K <= 24576.
 */
DGQ_API dgq_status dgq_rmsnorm_quant_act(const uint16_t *x, const uint16_t *gamma, int M, int K, float eps,
                                 int8_t *xq, float *sx, void *stream);
DGQ_API dgq_status dgq_silu_mul_quant_act(const uint16_t *gate_up, int M, int I, int8_t *xq, float *sx,
                                  void *stream);

/*
 * Static tensor-wise INT8 activation quantizer (the "S" scheme of Section 4.1 and Table 5;
 * symmetric form of Eq. 1): one positive scale for the whole tensor, fixed offline,
 *   xq = clamp(round(x / scale), -127, 127)   (one IEEE division per element, ties to even)
 * and sx[m] = scale for every token, so that dgq_linear_a8w4 takes the result unchanged.
 * Values beyond 127*scale saturate.  DGQ_ERR_RANGE unless 0 < scale < 3e38.
 */
DGQ_API dgq_status dgq_quant_act_static(const uint16_t *x, int M, int K, float scale, int8_t *xq, float *sx,
                                void *stream);

/*
 * Fused A8W4 linear: in-register INT4->INT8 expansion, INT8 MFMA GEMM with INT32
 * accumulation over all of K, scale epilogue (all three lines of Eq. 2):
 *   out[m][n] = fp16( (sx[m] * s1[n]) * (float) sum_k xq[m][k] * (s2[k/group][n] * w4[k][n]) )
 *   xq, sx            in  as written by dgq_quant_act
 *   qweight, scales   in  as written by dgq_pack_weights for the same K, N, group
 *   s1                in  [N] float
 *   out               out [M][N] fp16 (raw bits)
 *   workspace         scratch of at least dgq_linear_workspace_bytes(), zero-filled before
 *                     its first use (see the workspace contract above)
 * M <= 16 takes a weight-streaming split-K kernel, larger M a tiled MFMA kernel (64- or
 * 128-token tiles; K split over several workgroups per tile where the tiles alone would
 * leave compute units idle, the last workgroup to finish a tile adding up the parts); all
 * give the same INT32 sums.
 */
DGQ_API dgq_status dgq_linear_a8w4(const int8_t *xq, const float *sx, const void *qweight,
                           const void *scales, const float *s1, uint16_t *out,
                           int M, int N, int K, int group,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * dgq_linear_a8w4 for callers that can neither allocate device memory nor bring a workspace:
 * code recorded into a HIP graph, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments without the workspace, same kernels, same bits.  Where the problem needs scratch (the
 * INT32 partial sums of a K split, dgq_linear_workspace_bytes() > 0) it lives in a static device
 * array of 40 MiB inside the library, which every GPU the library has run on holds until the
 * process ends; a problem that needs more returns DGQ_ERR_WORKSPACE (nothing is launched).  The
 * call makes no hipMalloc / hipFree and no allocating library call.  The first call on a device
 * looks up that device's address of the array (hipGetSymbolAddress with the device current, as
 * for any launch); make that first call outside graph capture.  All calls on one GPU share the
 * array: calls that need scratch and may overlap on one GPU (different streams, or graph
 * branches) race and must be ordered by the caller.  The array starts out zero-filled and every
 * call leaves its arrival counters zero again, which is all the workspace contract asks for.
 */
DGQ_API dgq_status dgq_linear_a8w4_noalloc(const int8_t *xq, const float *sx, const void *qweight,
                                   const void *scales, const float *s1, uint16_t *out,
                                   int M, int N, int K, int group, void *stream);

/*
 * Test hook: same kernels and main loop as dgq_linear_a8w4 but the epilogue stores the
 * raw INT32 sums X_s8 W_s8 (third line of Eq. 2 before scaling) to acc_out [M][N].
 *   path  0 = the kernel dgq_linear_a8w4 chooses for this M; 1 = the weight-streaming
 *         kernels; 2 = the tiled kernel; 3 = the weight-streaming kernel that re-reads
 *         activations every step (never chosen by M; kept as an independent check, signed
 *         nibbles only).  The weight-streaming kernels take M <= 64 (DGQ_ERR_SHAPE beyond);
 *         any other value gives DGQ_ERR_RANGE.
 *   workspace  at least dgq_linear_acc_workspace_bytes() for the same path
 */
DGQ_API dgq_status dgq_linear_a8w4_acc(const int8_t *xq, const void *qweight, const void *scales,
                               int32_t *acc_out, int M, int N, int K, int group, int path,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * ---- General operands of Eq. 2: unsigned nibbles with per-group zero points --------------
 *
 * Section 3.2 lists the operands as W_u4 in [0, 15], group-wise zero points ZP and group-wise
 * INT8 scales S2, with W_s8 = S2 * (W_u4 - ZP) (sign as in Eq. 1 and Appendix B); Section 3.3
 * allows S2 above 15 as long as W_s8 fits INT8 (Eq. 4).  The calls below take that form:
 * S2 in [1, 127], ZP in [0, 15], every product S2 * (u - ZP) inside [-128, 127].  The calls
 * above are the special case ZP = 8, S2 <= 15 with a smaller scale array.
 *
 * Format: qweight as written by dgq_pack_weights, the stored nibble being W_u4 itself.
 * scales_zp: two bytes per (group, column), S2 then ZP, at
 * ((n/16)*ceil(ng/2) + gi/2)*64 + (n%16)*4 + (gi%2)*2; padding bytes are 0;
 * scales_zp_bytes = (N/16) * ceil((K/group)/2) * 64.
 */
DGQ_API dgq_status dgq_packed_sizes_zp(int K, int N, int group, size_t *qweight_bytes, size_t *scales_zp_bytes);

/*
 *   w_u4  in  [K][N] uint8, nibbles in [0, 15]
 *   s2    in  [K/group][N] uint8 in [1, 127];  zp in [K/group][N] uint8 in [0, 15]
 *   bad_count in/out, nullable, zeroed by the caller: the kernels add the number of rule
 *         breakers.  A scale outside its range is packed as 1, a zero point above 15 as 0, a
 *         nibble above 15 or with S2 * (u - ZP) outside [-128, 127] as ZP (a zero weight).
 */
DGQ_API dgq_status dgq_pack_weights_zp(const uint8_t *w_u4, const uint8_t *s2, const uint8_t *zp, int K, int N,
                               int group, void *qweight, void *scales_zp, int32_t *bad_count, void *stream);

/*
 * Two-phase grid search quantizer (Section 3.3, Eq. 3 to Eq. 5, clip of Eq. 4) with the
 * weight-only objective ||W - Q(W)||^2 (no calibration activations).  alpha runs over
 * 1, 1 - step, ..., 1 - (n_alpha - 1)*step, in both phases; the first minimum wins.
 *   phase 1, per group and column:  lo = min(min W, 0), hi = max(max W, 0),
 *       s = alpha*(hi - lo)/15, ZP = clamp(round(-(alpha*lo)/s), 0, 15),
 *       u = clamp(round(W/s) + ZP, 0, 15); the best alpha gives S' and ZP
 *   phase 2, per column:  s1 = alpha * max_j S'_j / 15, S2 = clamp(round(S'/s1), 1, 127),
 *       u = clamp(round(W/(s1*S2)) + ZP, ZP - floor(127/S2), ZP + floor(127/S2)) within [0, 15]
 * fp32, IEEE division, ties to even, sums in increasing k; an all-zero group gets S' = 0 and
 * ZP = 0, an all-zero column s1 = 1, S2 = 1.
 *   W      in  [K][N] fp16 (raw bits)
 *   w_u4   out [K][N] uint8;  zp, s2 out [K/group][N] uint8;  s1 out [N] float
 *   workspace  at least (K/group)*N*4 bytes (the S' of phase 1)
 * Errors: DGQ_ERR_RANGE if n_alpha is outside [1, 1024] or the smallest alpha is not positive.
 * The outputs are the inputs of dgq_pack_weights_zp.
 */
DGQ_API dgq_status dgq_quantize_weights_grid(const uint16_t *W, int K, int N, int group, int n_alpha, float step,
                                     uint8_t *w_u4, uint8_t *zp, uint8_t *s2, float *s1,
                                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same two-phase search with the activation-weighted objectives the paper states (Eq. 3 for
 * phase 1, the objective printed with Eq. 5 for phase 2), on calibration activations:
 *   phase 1, group j of column n:  err = sum_m ( X_j[m,:] w_j - Xh_j[m,:] Q(w_j) )^2
 *   phase 2, column n:             err = sum_m ( X[m,:] w     - Xh[m,:]  Q(w)   )^2
 * with Xh[m][k] = sx[m] * xq[m][k], the dequantized per-token INT8 form of X (xq, sx as written by
 * dgq_quant_act(X)).  Candidates, alpha grid, clip and tie rule as in dgq_quantize_weights_grid;
 * fp32, each product of a token summed on its own in increasing k, the squares in increasing m.
 *   W   in  [K][N] fp16;   X in [M][K] fp16, 1 <= M <= 4096 calibration tokens
 *   xq  in  [M][K] int8;   sx in [M] float
 *   outputs as for dgq_quantize_weights_grid
 *   workspace  at least dgq_quantize_weights_grid_act_workspace_bytes() (4 bytes times
 *              (K/group)*N + M*K + (K/group)*M*N + M*N)
 * Offline and written for clarity, not speed: the work grows with n_alpha * M * K * N.
 */
DGQ_API dgq_status dgq_quantize_weights_grid_act_workspace_bytes(int M, int K, int N, int group, size_t *bytes);
DGQ_API dgq_status dgq_quantize_weights_grid_act(const uint16_t *W, const uint16_t *X, const int8_t *xq, const float *sx,
                                         int M, int K, int N, int group, int n_alpha, float step,
                                         uint8_t *w_u4, uint8_t *zp, uint8_t *s2, float *s1,
                                         void *workspace, size_t workspace_bytes, void *stream);

/* Test hook: W_s8[K][N] = S2 * (W_u4 - ZP) from the packed form. */
DGQ_API dgq_status dgq_unpack_weights_zp(const void *qweight, const void *scales_zp, int K, int N, int group,
                                 int8_t *w_s8, void *stream);

/*
 * dgq_linear_a8w4 / dgq_linear_a8w4_acc for operands packed by dgq_pack_weights_zp: same
 * kernels (the zero point is one more byte in the scale word), same arguments, same workspace
 * rule.  path 3 of the test hook is not available for this form (DGQ_ERR_SHAPE).
 */
DGQ_API dgq_status dgq_linear_a8w4_zp(const int8_t *xq, const float *sx, const void *qweight,
                              const void *scales_zp, const float *s1, uint16_t *out,
                              int M, int N, int K, int group,
                              void *workspace, size_t workspace_bytes, void *stream);
DGQ_API dgq_status dgq_linear_a8w4_zp_acc(const int8_t *xq, const void *qweight, const void *scales_zp,
                                  int32_t *acc_out, int M, int N, int K, int group, int path,
                                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * dgq_quant_act followed by dgq_linear_a8w4 (dgq_linear_a8w4_zp) as one call: the per-token
 * dynamic quantizer of Section 3.1 / 4.1 in front of all three lines of Eq. 2,
 *   out = linear_a8w4(quant_act(x)),
 * with the same bits as the two calls.
 *   x          in  [M][K] fp16 (raw bits)
 *   qweight, scales (scales_zp), s1, out, M, N, K, group: as for dgq_linear_a8w4(_zp)
 *   sx_out     out [M] float, optional (may be NULL): the token scales the quantizer derived
 *   workspace  scratch of at least dgq_quant_linear_workspace_bytes(); may be NULL when
 *              that is 0
 * For M <= 16, K <= 12288 and M * (K + 16) <= 49152 (up to four tokens of a LLaMA-7B layer)
 * ONE kernel does both: every workgroup of the weight-streaming kernel needs whole token rows
 * anyway, so its threads share out the quantizer's work while the first weight loads are in
 * flight and hand the INT8 rows on through LDS; xq and sx never go through memory and the
 * second launch disappears.  Every workgroup repeats the quantizer, which is why this is limited
 * to small M * K.  Otherwise the call enqueues the two kernels with xq and sx placed in the
 * workspace.  dgq_quant_linear_plan names the GEMM kernel as
 * dgq_linear_plan does ("quant_linear_decode_kernel<2, 2, 128>" for the one-kernel form).
 * Errors as for dgq_quant_act and dgq_linear_a8w4.
 */
DGQ_API dgq_status dgq_quant_linear_workspace_bytes(int M, int N, int K, int group, size_t *bytes);
DGQ_API dgq_status dgq_quant_linear_a8w4(const uint16_t *x, const void *qweight, const void *scales,
                                 const float *s1, uint16_t *out, float *sx_out, int M, int N, int K,
                                 int group, void *workspace, size_t workspace_bytes, void *stream);
DGQ_API dgq_status dgq_quant_linear_a8w4_zp(const uint16_t *x, const void *qweight, const void *scales_zp,
                                    const float *s1, uint16_t *out, float *sx_out, int M, int N, int K,
                                    int group, void *workspace, size_t workspace_bytes, void *stream);
DGQ_API dgq_status dgq_quant_linear_plan(int M, int N, int K, int group, char *buf, size_t buf_bytes);

/*
 * dgq_rmsnorm_quant_act followed by dgq_linear_a8w4 (dgq_linear_a8w4_zp) as one call: the
 * producer of a transformer block's first linears (qkv, gate+up), the per-token quantizer and
 * Eq. 2,
 *   out = linear_a8w4(quant_act(rmsnorm(x) * gamma)),
 * with y = fp16(float(x * (1 / sqrt(mean_k x^2 + eps)) * gamma[k])) evaluated in fp64 as in
 * dgq_rmsnorm_quant_act.  Arguments as for dgq_quant_linear_a8w4, plus
 *   gamma  in [K] fp16 (raw bits), 16-byte aligned;   0 <= eps < 1 (DGQ_ERR_RANGE otherwise)
 * K <= 24576.  One kernel under the conditions of dgq_quant_linear_a8w4 and K <= 8192 (the
 * hidden sizes of LLaMA-7B to 65B); otherwise the two kernels, with xq and sx in the workspace
 * (dgq_rmsnorm_quant_linear_workspace_bytes).  Both forms add the squares in the same fixed order,
 * so they give the same bits.
 */
DGQ_API dgq_status dgq_rmsnorm_quant_linear_workspace_bytes(int M, int N, int K, int group, size_t *bytes);
DGQ_API dgq_status dgq_rmsnorm_quant_linear_a8w4(const uint16_t *x, const uint16_t *gamma, float eps,
                                         const void *qweight, const void *scales, const float *s1,
                                         uint16_t *out, float *sx_out, int M, int N, int K, int group,
                                         void *workspace, size_t workspace_bytes, void *stream);
DGQ_API dgq_status dgq_rmsnorm_quant_linear_a8w4_zp(const uint16_t *x, const uint16_t *gamma, float eps,
                                            const void *qweight, const void *scales_zp, const float *s1,
                                            uint16_t *out, float *sx_out, int M, int N, int K, int group,
                                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * Batched INT8 matrix product for attention.  Section 4.1 ("Implementation") runs the attention
 * products as INT8 batched matrix multiplications and says no more; taken here as: both operands
 * INT8 with the reduction index contiguous, one INT32 sum over all of K, and the scale epilogue of
 * Eq. 2 (first and third line) with the second operand's per-token scale in the place of the
 * channel scale, rounded once to fp16:
 *   out[i][m][n] = fp16( (sa[i][m] * sb[i][n]) * (float) sum_k a[i][m][k] * b[i][n][k] )
 * (attention scores: a = Q, b = K; context: a = P, b = V transposed).
 *   a    in  [batch][M][K] int8;   b  in  [batch][N][K] int8
 *   sa   in  [batch][M] float, sb in [batch][N] float; either may be NULL (= all ones); a static
 *        tensor-wise scale is an array filled with that scale
 *   out  out [batch][M][N] fp16 (raw bits)
 * Shape rules: 1 <= batch <= 65535, M, N >= 1 (any values; 16-byte stores are used when N % 8 == 0),
 * K % 16 == 0, 16 <= K <= 65536 (INT32 sums cannot wrap).  No workspace.
 * dgq_bmm_s8_acc is the test hook that stores the raw INT32 sums [batch][M][N].
 */
DGQ_API dgq_status dgq_bmm_s8(const int8_t *a, const int8_t *b, const float *sa, const float *sb, uint16_t *out,
                      int batch, int M, int N, int K, void *stream);
DGQ_API dgq_status dgq_bmm_s8_acc(const int8_t *a, const int8_t *b, int32_t *acc_out, int batch, int M, int N, int K,
                          void *stream);

/*
 * Measurement aid (host function, nothing launched): writes into buf (at least 96 bytes)
 * the name, with template arguments, of the GEMM kernel that dgq_linear_a8w4 would launch
 * for this problem, e.g. "linear_decode_kernel<2, 2, 128, false, false>".  Profiler output can be matched to it.
 */
DGQ_API dgq_status dgq_linear_plan(int M, int N, int K, int group, char *buf, size_t buf_bytes);

/*
 * Measurement aid (not part of Eq. 2): reads `bytes` (a multiple of 16 is read, the rest is
 * ignored) of a device buffer once with `workgroups` 1024-thread workgroups and 128-bit
 * loads, the access pattern of the weight stream.  `sink` is a device array of `workgroups`
 * uint32 that is written only in the unlikely case a checksum matches; it exists so that the
 * loads cannot be optimised away.  Timing this call gives the read bandwidth a
 * weight-streaming kernel could at best reach for a buffer of that size.
 */
DGQ_API dgq_status dgq_probe_read(const void *src, size_t bytes, uint32_t *sink, int workgroups, void *stream);

/*
 * Measurement aid (not part of Eq. 2): every lane of `workgroups` 256-thread workgroups takes
 * six 16-byte MFMA operands from `operands` (`bytes` >= 96; lane l reads 96 bytes at offset
 * 96*l, wrapping around) and issues 8*iters v_mfma_i32_32x32x32_i8 on them with no memory
 * access in the loop: 2*32*32*32 * 8 * iters * 4 * workgroups integer operations in all.  The
 * matrix-core rate depends on the operand data (the chip lowers its clock with switching
 * activity), so timing this call on a buffer of real INT8 activations or expanded weights
 * gives the ceiling that applies to the GEMM of Eq. 2 on such data; a zeroed buffer gives
 * the data-independent peak.  `sink`: as for dgq_probe_read.
 */
DGQ_API dgq_status dgq_probe_mfma(const void *operands, size_t bytes, int iters, uint32_t *sink,
                          int workgroups, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DGQ_H */
