/*
 * CPU oracle for the Dual Grained Quantization (DGQ) A8W4 linear layer.
 *
 * TEST INFRASTRUCTURE, NOT THE PRODUCT.  Plain scalar loops, no blocking, no
 * intrinsics.  It shares no code with the HIP path and is only ever called by
 * the tests, the smoke check and the benchmark's cpu_baseline leg.
 *
 * Orientation follows the paper (Section 3.2): activations X are [M][K]
 * (b x h), weights are [K][N] (h x o, N contiguous), groups of `g` consecutive
 * input channels k share one integer scale per output channel n.
 *
 * Floating-point values cross this boundary as fp32; fp16 inputs are widened
 * exactly by the caller and the final fp16 rounding of the output is one
 * round-to-nearest-even conversion done by the caller.
 *
 * Every loop that is parallelised with OpenMP iterates over independent
 * outputs; no arithmetic is reordered by it.
 *
 * Parity status: every function below is pinned by tests that do not go
 * through this file's own formulas (hand-written tiny cases, closed forms,
 * numpy int64 matmul, an fp64 group-wise "segmented GEMM"; for the grid search:
 * exactly representable inputs that it must recover, a brute-force check of the
 * Eq. 4 interval, the min-max special case, error bounds; for the batched product: a hand-worked
 * case, numpy int64, one-hot operands, and the already pinned GEMM on a transposed operand).  The statistical
 * accuracy of the RTN and grid-search quantizers against the paper's perplexity
 * tables is parity unpinned (needs the trained models and datasets).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int dgq_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static float clampf(float v, float lo, float hi) { return v < lo ? lo : (v > hi ? hi : v); }

/*
 * Round-to-nearest dual-grained weight quantizer (the "RTN" row of Table 1;
 * symmetric scale of Section 3.1; scale decoupling S = s1 * S2 of Eq. 5).
 *
 *   S'[j][n] = max_{k in group j} |W[k][n]| / 7            (4-bit symmetric)
 *   s1[n]    = max_j S'[j][n] / 15
 *   s2[j][n] = clamp(round(S'[j][n] / s1[n]), 1, 15)
 *   w4[k][n] = clamp(round(W[k][n] / (s1[n] * s2[j][n])), -8, 7)
 *
 * All in fp32, one IEEE division where a '/' is written, ties to even.
 * An all-zero column gets s1 = 1, s2 = 1, w4 = 0.
 */
void dgq_oracle_quantize_rtn(const float *W, int K, int N, int g,
                             int8_t *w4, uint8_t *s2, float *s1)
{
    const int ng = K / g;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        float spmax = 0.0f;
        for (int j = 0; j < ng; ++j) {
            float a = 0.0f;
            for (int k = j * g; k < (j + 1) * g; ++k) {
                float v = fabsf(W[(size_t)k * N + n]);
                if (v > a) a = v;
            }
            float sp = a / 7.0f;
            if (sp > spmax) spmax = sp;
        }
        if (spmax == 0.0f) {
            s1[n] = 1.0f;
            for (int j = 0; j < ng; ++j) s2[(size_t)j * N + n] = 1;
            for (int k = 0; k < K; ++k) w4[(size_t)k * N + n] = 0;
            continue;
        }
        const float c = spmax / 15.0f;
        s1[n] = c;
        for (int j = 0; j < ng; ++j) {
            float a = 0.0f;
            for (int k = j * g; k < (j + 1) * g; ++k) {
                float v = fabsf(W[(size_t)k * N + n]);
                if (v > a) a = v;
            }
            float sp = a / 7.0f;
            float q = clampf(rintf(sp / c), 1.0f, 15.0f);
            s2[(size_t)j * N + n] = (uint8_t)q;
            float S = c * q;
            for (int k = j * g; k < (j + 1) * g; ++k) {
                float w = clampf(rintf(W[(size_t)k * N + n] / S), -8.0f, 7.0f);
                w4[(size_t)k * N + n] = (int8_t)w;
            }
        }
    }
}

/*
 * Per-token dynamic symmetric INT8 activation quantizer (Section 3.1,
 * symmetric case with N = 8 bits; "per-token dynamic" of Section 4.1):
 *
 *   a     = max_k |x[m][k]|
 *   sx[m] = a / 127
 *   xq    = clamp(round(x * (127 / a)), -127, 127)
 *
 * fp32, ties to even.  A zero row gives sx = 0 and xq = 0.
 */
void dgq_oracle_quant_act(const float *x, int M, int K, int8_t *xq, float *sx)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        const float *row = x + (size_t)m * K;
        float a = 0.0f;
        for (int k = 0; k < K; ++k) {
            float v = fabsf(row[k]);
            if (v > a) a = v;
        }
        if (a == 0.0f) {
            sx[m] = 0.0f;
            memset(xq + (size_t)m * K, 0, (size_t)K);
            continue;
        }
        sx[m] = a / 127.0f;
        const float inv = 127.0f / a;
        for (int k = 0; k < K; ++k) {
            float q = clampf(rintf(row[k] * inv), -127.0f, 127.0f);
            xq[(size_t)m * K + k] = (int8_t)q;
        }
    }
}

/*
 * INT4 -> INT8 expansion, second line of Eq. 2 with the zero point folded
 * into the signed nibble:  W_s8[k][n] = s2[k/g][n] * w4[k][n].
 * Returns how many products fall outside [-128, 127] (the range constraint
 * stated next to Eq. 4); those entries are stored saturated.
 */
long dgq_oracle_expand(const int8_t *w4, const uint8_t *s2, int K, int N, int g, int8_t *ws8)
{
    long bad = 0;
#pragma omp parallel for schedule(static) reduction(+ : bad)
    for (int k = 0; k < K; ++k) {
        for (int n = 0; n < N; ++n) {
            int v = (int)s2[(size_t)(k / g) * N + n] * (int)w4[(size_t)k * N + n];
            if (v < -128 || v > 127) {
                ++bad;
                v = v < -128 ? -128 : 127;
            }
            ws8[(size_t)k * N + n] = (int8_t)v;
        }
    }
    return bad;
}

/*
 * INT8 x INT8 -> INT32 GEMM, one unbroken reduction over all of K (third line
 * of Eq. 2):  acc[m][n] = sum_k xq[m][k] * ws8[k][n].
 * A 64-bit shadow sum checks that INT32 never wraps; returns the number of
 * outputs where it would have.
 */
long dgq_oracle_gemm_i32(const int8_t *xq, const int8_t *ws8, int M, int N, int K, int32_t *acc)
{
    long wrapped = 0;
#pragma omp parallel for schedule(static) reduction(+ : wrapped)
    for (int n = 0; n < N; ++n) {
        for (int m = 0; m < M; ++m) {
            int32_t a32 = 0;
            int64_t a64 = 0;
            for (int k = 0; k < K; ++k) {
                int p = (int)xq[(size_t)m * K + k] * (int)ws8[(size_t)k * N + n];
                a32 = (int32_t)((uint32_t)a32 + (uint32_t)p);
                a64 += p;
            }
            if ((int64_t)a32 != a64) ++wrapped;
            acc[(size_t)m * N + n] = a32;
        }
    }
    return wrapped;
}

/*
 * Batched INT8 x INT8 -> INT32 matrix product for attention (Section 4.1, "Implementation": the
 * attention products run as INT8 batched matrix multiplications; the paper gives no more than
 * that).  Both operands have the reduction index contiguous:
 *     acc[b][m][n] = sum_k A[b][m][k] * B[b][n][k]
 * (scores: A = Q, B = K; context: A = P, B = V transposed), one unbroken INT32 sum over all of K
 * with a 64-bit shadow sum; returns the number of outputs that would wrap.  The scale epilogue
 * is the one of Eq. 2 (dgq_oracle_epilogue per batch) with the two operands' per-token scales.
 */
long dgq_oracle_bmm_s8(const int8_t *A, const int8_t *B, int batch, int M, int N, int K, int32_t *acc)
{
    long wrapped = 0;
#pragma omp parallel for schedule(static) reduction(+ : wrapped) collapse(2)
    for (int b = 0; b < batch; ++b) {
        for (int m = 0; m < M; ++m) {
            const int8_t *a = A + ((size_t)b * M + m) * K;
            for (int n = 0; n < N; ++n) {
                const int8_t *w = B + ((size_t)b * N + n) * K;
                int32_t a32 = 0;
                int64_t a64 = 0;
                for (int k = 0; k < K; ++k) {
                    const int p = (int)a[k] * (int)w[k];
                    a32 = (int32_t)((uint32_t)a32 + (uint32_t)p);
                    a64 += p;
                }
                if ((int64_t)a32 != a64) ++wrapped;
                acc[((size_t)b * M + m) * N + n] = a32;
            }
        }
    }
    return wrapped;
}

/*
 * Epilogue, first and third lines of Eq. 2: the per-token activation scale
 * times the per-output-channel weight scale, applied to the integer sum:
 *   out[m][n] = (sx[m] * s1[n]) * (float)acc[m][n]       (fp32)
 * The caller rounds out32 once to fp16.
 */
void dgq_oracle_epilogue(const int32_t *acc, const float *sx, const float *s1, int M, int N,
                         float *out32)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            float s = sx[m] * s1[n];
            out32[(size_t)m * N + n] = s * (float)acc[(size_t)m * N + n];
        }
    }
}

/*
 * Device weight format, written from the layout text alone.
 *
 *   stored nibble u = w4 + 8 (zero point 8), 0..15.
 *   qweight is a sequence of 16-byte cells.  Element (k, n) lives in cell
 *     ((n/16) * (K/128) + k/128) * 64 + ((k%128)/32) * 16 + n%16,
 *   in byte k%16 of that cell, low nibble when k%32 < 16, high nibble otherwise.
 *   scales holds one byte per (group, column):
 *     ((n/16) * ceil(ng/4) + gi/4) * 64 + (n%16) * 4 + gi%4,   gi = k/g,
 *   padding bytes (gi >= ng) are zero.
 *
 * Requires K % 128 == 0, N % 16 == 0, g in {64, 128}.  Returns the number of
 * inputs that break a range rule (nibble outside [-8,7], scale outside [1,15]);
 * such entries are packed as zero weight / scale 1.  Inside those ranges
 * |s2*w4| <= 120, so the INT8 constraint on the expanded weight always holds.
 */
long dgq_oracle_pack(const int8_t *w4, const uint8_t *s2, int K, int N, int g,
                     uint8_t *qweight, uint8_t *scales)
{
    const int ng = K / g;
    const int gq = (ng + 3) / 4;
    const int ksteps = K / 128;
    long bad = 0;
    memset(qweight, 0, (size_t)K * N / 2);
    memset(scales, 0, (size_t)(N / 16) * gq * 64);
    for (int gi = 0; gi < ng; ++gi) {
        for (int n = 0; n < N; ++n) {
            int s = s2[(size_t)gi * N + n];
            if (s < 1 || s > 15) {
                ++bad;
                s = 1;
            }
            scales[((size_t)(n / 16) * gq + gi / 4) * 64 + (size_t)(n % 16) * 4 + gi % 4] = (uint8_t)s;
        }
    }
    for (int k = 0; k < K; ++k) {
        for (int n = 0; n < N; ++n) {
            int w = w4[(size_t)k * N + n];
            if (w < -8 || w > 7) {
                ++bad;
                w = 0;
            }
            unsigned u = (unsigned)(w + 8);
            size_t cell = ((size_t)(n / 16) * ksteps + k / 128) * 64 + (size_t)((k % 128) / 32) * 16 + n % 16;
            size_t byte = cell * 16 + k % 16;
            if (k % 32 < 16)
                qweight[byte] |= (uint8_t)u;
            else
                qweight[byte] |= (uint8_t)(u << 4);
        }
    }
    return bad;
}

/* Inverse of dgq_oracle_pack: recovers w4 [K][N] and s2 [ng][N]. */
void dgq_oracle_unpack(const uint8_t *qweight, const uint8_t *scales, int K, int N, int g,
                       int8_t *w4, uint8_t *s2)
{
    const int ng = K / g;
    const int gq = (ng + 3) / 4;
    const int ksteps = K / 128;
    for (int gi = 0; gi < ng; ++gi)
        for (int n = 0; n < N; ++n)
            s2[(size_t)gi * N + n] =
                scales[((size_t)(n / 16) * gq + gi / 4) * 64 + (size_t)(n % 16) * 4 + gi % 4];
    for (int k = 0; k < K; ++k) {
        for (int n = 0; n < N; ++n) {
            size_t cell = ((size_t)(n / 16) * ksteps + k / 128) * 64 + (size_t)((k % 128) / 32) * 16 + n % 16;
            uint8_t b = qweight[cell * 16 + k % 16];
            unsigned u = (k % 32 < 16) ? (b & 15u) : (b >> 4);
            w4[(size_t)k * N + n] = (int8_t)((int)u - 8);
        }
    }
}

/* ======================================================================================
 * General form of the weight operands: unsigned nibbles with per-group zero points
 * (operands of Eq. 2 as Section 3.2 lists them), the overflow-safe clip of Eq. 4 and the
 * two-phase grid search of Section 3.3.
 * ====================================================================================== */

/*
 * Second line of Eq. 2 with an explicit zero point, in the sign convention of Eq. 1 and
 * Appendix B:  W_s8[k][n] = S2[k/g][n] * (W_u4[k][n] - ZP[k/g][n]).
 * Returns how many results fall outside [-128, 127]; those are stored saturated.
 */
long dgq_oracle_expand_zp(const uint8_t *u4, const uint8_t *s2, const uint8_t *zp, int K, int N, int g,
                          int8_t *ws8)
{
    long bad = 0;
#pragma omp parallel for schedule(static) reduction(+ : bad)
    for (int k = 0; k < K; ++k) {
        for (int n = 0; n < N; ++n) {
            const size_t gi = (size_t)(k / g) * N + n;
            int v = (int)s2[gi] * ((int)u4[(size_t)k * N + n] - (int)zp[gi]);
            if (v < -128 || v > 127) {
                ++bad;
                v = v < -128 ? -128 : 127;
            }
            ws8[(size_t)k * N + n] = (int8_t)v;
        }
    }
    return bad;
}

/*
 * Interval of Eq. 4: the stored nibbles u for which S2 * (u - ZP) stays inside
 * [-127, 127], intersected with [0, 15].  The quotient 127 / S2 is truncated (the paper
 * prints a rounding bracket; rounding it up would admit a product above 127, which is
 * what the interval exists to prevent).
 */
void dgq_oracle_clip_interval(int s2, int zp, int *lo, int *hi)
{
    const int r = 127 / s2;
    *lo = zp - r < 0 ? 0 : zp - r;
    *hi = zp + r > 15 ? 15 : zp + r;
}


/*
 * Two-phase grid search (Section 3.3) with the weight-only objective ||W - Q(W)||^2 (the
 * activations of Eq. 3 and of the phase-2 objective are taken as the identity: there is no
 * calibration set).  alpha runs over 1, 1 - step, ..., 1 - (n_alpha-1)*step.
 *
 * Phase 1, for every group j and column n on its own (Eq. 3, quantizer of Eq. 1 with
 * N = 4 bits):
 *     lo = min(min_k W, 0), hi = max(max_k W, 0)         the range always contains zero
 *     s  = alpha * (hi - lo) / 15,  ZP = clamp(round(-(alpha * lo) / s), 0, 15)
 *     u  = clamp(round(W / s) + ZP, 0, 15),  err = sum_k (W - (u - ZP) * s)^2
 *   the alpha with the smallest err (the first one on ties) gives S'[j][n] and ZP[j][n];
 *   an all-zero group gets S' = 0 and ZP = 0.
 *
 * Phase 2, for every column n (Eq. 5, clip of Eq. 4):
 *     s1 = alpha * max_j S'[j][n] / 15
 *     S2[j] = clamp(round(S'[j] / s1), 1, 127),  S = s1 * S2[j]
 *     u = clamp(round(W / S) + ZP[j], lo4, hi4) with [lo4, hi4] from dgq_oracle_clip_interval
 *     err = sum over the whole column of (W - (u - ZP) * S)^2
 *   the alpha with the smallest err (first on ties) gives s1[n], S2[:, n] and u4[:, n];
 *   an all-zero column gets s1 = 1, S2 = 1, u = ZP = 0.
 *
 * fp32 throughout, one IEEE division where a '/' is written, ties to even, sums in
 * increasing k.  W is [K][N]; u4 [K][N]; zp, s2 [K/g][N]; s1 [N].
 */
void dgq_oracle_quantize_grid(const float *W, int K, int N, int g, int n_alpha, float step,
                              uint8_t *u4, uint8_t *zp, uint8_t *s2, float *s1)
{
    const int ng = K / g;
#pragma omp parallel for schedule(dynamic, 4)
    for (int n = 0; n < N; ++n) {
        float *Sp = (float *)malloc(sizeof(float) * (size_t)ng);
        /* ---- phase 1 ---- */
        for (int j = 0; j < ng; ++j) {
            float lo = 0.0f, hi = 0.0f;
            for (int k = j * g; k < (j + 1) * g; ++k) {
                const float w = W[(size_t)k * N + n];
                if (w < lo) lo = w;
                if (w > hi) hi = w;
            }
            float best_err = 0.0f, best_s = 0.0f;
            int best_zp = 0, have = 0;
            if (hi - lo > 0.0f) {
                for (int i = 0; i < n_alpha; ++i) {
                    const float alpha = 1.0f - (float)i * step;
                    const float s = (alpha * (hi - lo)) / 15.0f;
                    const float z = clampf(rintf(-(alpha * lo) / s), 0.0f, 15.0f);
                    float err = 0.0f;
                    for (int k = j * g; k < (j + 1) * g; ++k) {
                        const float w = W[(size_t)k * N + n];
                        const float u = clampf(rintf(w / s) + z, 0.0f, 15.0f);
                        const float d = w - (u - z) * s;
                        err = err + d * d;
                    }
                    if (!have || err < best_err) {
                        have = 1;
                        best_err = err;
                        best_s = s;
                        best_zp = (int)z;
                    }
                }
            }
            Sp[j] = best_s;
            zp[(size_t)j * N + n] = (uint8_t)best_zp;
        }
        /* ---- phase 2 ---- */
        float smax = 0.0f;
        for (int j = 0; j < ng; ++j)
            if (Sp[j] > smax) smax = Sp[j];
        if (!(smax > 0.0f)) {
            s1[n] = 1.0f;
            for (int j = 0; j < ng; ++j) s2[(size_t)j * N + n] = 1, zp[(size_t)j * N + n] = 0;
            for (int k = 0; k < K; ++k) u4[(size_t)k * N + n] = 0;
            free(Sp);
            continue;
        }
        float best_err = 0.0f, best_s1 = 0.0f;
        int have = 0;
        for (int i = 0; i < n_alpha; ++i) {
            const float alpha = 1.0f - (float)i * step;
            const float c1 = (alpha * smax) / 15.0f;
            float err = 0.0f;
            for (int j = 0; j < ng; ++j) {
                const float q2 = clampf(rintf(Sp[j] / c1), 1.0f, 127.0f);
                const float S = c1 * q2;
                const int z = zp[(size_t)j * N + n];
                int lo4, hi4;
                dgq_oracle_clip_interval((int)q2, z, &lo4, &hi4);
                for (int k = j * g; k < (j + 1) * g; ++k) {
                    const float w = W[(size_t)k * N + n];
                    const float u = clampf(rintf(w / S) + (float)z, (float)lo4, (float)hi4);
                    const float d = w - (u - (float)z) * S;
                    err = err + d * d;
                }
            }
            if (!have || err < best_err) {
                have = 1;
                best_err = err;
                best_s1 = c1;
            }
        }
        s1[n] = best_s1;
        for (int j = 0; j < ng; ++j) {
            const float q2 = clampf(rintf(Sp[j] / best_s1), 1.0f, 127.0f);
            const float S = best_s1 * q2;
            const int z = zp[(size_t)j * N + n];
            int lo4, hi4;
            dgq_oracle_clip_interval((int)q2, z, &lo4, &hi4);
            s2[(size_t)j * N + n] = (uint8_t)q2;
            for (int k = j * g; k < (j + 1) * g; ++k) {
                const float w = W[(size_t)k * N + n];
                const float u = clampf(rintf(w / S) + (float)z, (float)lo4, (float)hi4);
                u4[(size_t)k * N + n] = (uint8_t)u;
            }
        }
        free(Sp);
    }
}

/*
 * Two-phase grid search with the activation-weighted objectives of Section 3.3 (Eq. 3 for
 * phase 1, the objective printed with Eq. 5 for phase 2), on calibration activations X [M][K]
 * and their dequantized form Xh [M][K] (the per-token INT8 quantization of X times its scale):
 *
 *   phase 1, group j of column n:   err = sum_m ( X_j[m,:] w_j  -  Xh_j[m,:] Q(w_j) )^2
 *   phase 2, column n:              err = sum_m ( X[m,:] w      -  Xh[m,:]  Q(w)   )^2
 *
 * where X_j, w_j are the K-slice of group j.  Everything else (alpha grid, scale and zero point
 * of a candidate, S2, the Eq. 4 clip, first minimum wins, zero groups and columns) is as in
 * dgq_oracle_quantize_grid.  fp32; each of the two products of a token is summed on its own in
 * increasing k, then subtracted; the squares are added in increasing m.
 */
static float weighted_err(const float *Xh, int M, int K, int k0, int k1, const float *xw, const float *wq)
{
    float err = 0.0f;
    for (int m = 0; m < M; ++m) {
        float t = 0.0f;
        for (int k = k0; k < k1; ++k) t = t + Xh[(size_t)m * K + k] * wq[k - k0];
        const float d = xw[m] - t;
        err = err + d * d;
    }
    return err;
}

void dgq_oracle_quantize_grid_act(const float *W, const float *X, const float *Xh, int M, int K, int N, int g,
                                  int n_alpha, float step, uint8_t *u4, uint8_t *zp, uint8_t *s2, float *s1)
{
    const int ng = K / g;
#pragma omp parallel for schedule(dynamic, 4)
    for (int n = 0; n < N; ++n) {
        float *Sp = (float *)malloc(sizeof(float) * (size_t)ng);
        float *xw = (float *)malloc(sizeof(float) * (size_t)M);     /* X w of the slice in hand, per token */
        float *wq = (float *)malloc(sizeof(float) * (size_t)K);     /* dequantized candidate */
        /* ---- phase 1 ---- */
        for (int j = 0; j < ng; ++j) {
            const int k0 = j * g, k1 = (j + 1) * g;
            float lo = 0.0f, hi = 0.0f;
            for (int k = k0; k < k1; ++k) {
                const float w = W[(size_t)k * N + n];
                if (w < lo) lo = w;
                if (w > hi) hi = w;
            }
            float best_err = 0.0f, best_s = 0.0f;
            int best_zp = 0, have = 0;
            if (hi - lo > 0.0f) {
                for (int m = 0; m < M; ++m) {
                    float t = 0.0f;
                    for (int k = k0; k < k1; ++k) t = t + X[(size_t)m * K + k] * W[(size_t)k * N + n];
                    xw[m] = t;
                }
                for (int i = 0; i < n_alpha; ++i) {
                    const float alpha = 1.0f - (float)i * step;
                    const float s = (alpha * (hi - lo)) / 15.0f;
                    const float z = clampf(rintf(-(alpha * lo) / s), 0.0f, 15.0f);
                    for (int k = k0; k < k1; ++k) {
                        const float u = clampf(rintf(W[(size_t)k * N + n] / s) + z, 0.0f, 15.0f);
                        wq[k - k0] = (u - z) * s;
                    }
                    const float err = weighted_err(Xh, M, K, k0, k1, xw, wq);
                    if (!have || err < best_err) {
                        have = 1;
                        best_err = err;
                        best_s = s;
                        best_zp = (int)z;
                    }
                }
            }
            Sp[j] = best_s;
            zp[(size_t)j * N + n] = (uint8_t)best_zp;
        }
        /* ---- phase 2 ---- */
        float smax = 0.0f;
        for (int j = 0; j < ng; ++j)
            if (Sp[j] > smax) smax = Sp[j];
        if (!(smax > 0.0f)) {
            s1[n] = 1.0f;
            for (int j = 0; j < ng; ++j) s2[(size_t)j * N + n] = 1, zp[(size_t)j * N + n] = 0;
            for (int k = 0; k < K; ++k) u4[(size_t)k * N + n] = 0;
            free(Sp), free(xw), free(wq);
            continue;
        }
        for (int m = 0; m < M; ++m) {
            float t = 0.0f;
            for (int k = 0; k < K; ++k) t = t + X[(size_t)m * K + k] * W[(size_t)k * N + n];
            xw[m] = t;
        }
        float best_err = 0.0f, best_s1 = 0.0f;
        int have = 0;
        for (int i = 0; i < n_alpha; ++i) {
            const float alpha = 1.0f - (float)i * step;
            const float c1 = (alpha * smax) / 15.0f;
            for (int j = 0; j < ng; ++j) {
                const float q2 = clampf(rintf(Sp[j] / c1), 1.0f, 127.0f);
                const float S = c1 * q2;
                const int z = zp[(size_t)j * N + n];
                int lo4, hi4;
                dgq_oracle_clip_interval((int)q2, z, &lo4, &hi4);
                for (int k = j * g; k < (j + 1) * g; ++k) {
                    const float u = clampf(rintf(W[(size_t)k * N + n] / S) + (float)z, (float)lo4, (float)hi4);
                    wq[k] = (u - (float)z) * S;
                }
            }
            const float err = weighted_err(Xh, M, K, 0, K, xw, wq);
            if (!have || err < best_err) {
                have = 1;
                best_err = err;
                best_s1 = c1;
            }
        }
        s1[n] = best_s1;
        for (int j = 0; j < ng; ++j) {
            const float q2 = clampf(rintf(Sp[j] / best_s1), 1.0f, 127.0f);
            const float S = best_s1 * q2;
            const int z = zp[(size_t)j * N + n];
            int lo4, hi4;
            dgq_oracle_clip_interval((int)q2, z, &lo4, &hi4);
            s2[(size_t)j * N + n] = (uint8_t)q2;
            for (int k = j * g; k < (j + 1) * g; ++k) {
                const float u = clampf(rintf(W[(size_t)k * N + n] / S) + (float)z, (float)lo4, (float)hi4);
                u4[(size_t)k * N + n] = (uint8_t)u;
            }
        }
        free(Sp), free(xw), free(wq);
    }
}

/*
 * Device format for the general operands, written from the layout text alone.
 *   qweight: as in dgq_oracle_pack, the stored nibble being W_u4 itself.
 *   scales_zp: two bytes per (group, column), the group scale S2 then the zero point, at
 *     ((n/16) * ceil(ng/2) + gi/2) * 64 + (n%16) * 4 + (gi%2) * 2;   padding bytes are zero.
 * Returns the number of inputs that break a rule: S2 outside [1, 127] (packed as 1), ZP
 * above 15 (packed as 0), a nibble above 15 or a product S2 * (u - ZP) outside [-128, 127]
 * (the nibble is then packed as ZP, a zero weight).
 */
long dgq_oracle_pack_zp(const uint8_t *u4, const uint8_t *s2, const uint8_t *zp, int K, int N, int g,
                        uint8_t *qweight, uint8_t *scales_zp)
{
    const int ng = K / g;
    const int gh = (ng + 1) / 2;
    const int ksteps = K / 128;
    long bad = 0;
    memset(qweight, 0, (size_t)K * N / 2);
    memset(scales_zp, 0, (size_t)(N / 16) * gh * 64);
    for (int gi = 0; gi < ng; ++gi) {
        for (int n = 0; n < N; ++n) {
            int s = s2[(size_t)gi * N + n], z = zp[(size_t)gi * N + n];
            if (s < 1 || s > 127) {
                ++bad;
                s = 1;
            }
            if (z > 15) {
                ++bad;
                z = 0;
            }
            const size_t at = ((size_t)(n / 16) * gh + gi / 2) * 64 + (size_t)(n % 16) * 4 + (size_t)(gi % 2) * 2;
            scales_zp[at] = (uint8_t)s;
            scales_zp[at + 1] = (uint8_t)z;
        }
    }
    for (int k = 0; k < K; ++k) {
        for (int n = 0; n < N; ++n) {
            const int gi = k / g;
            int s = s2[(size_t)gi * N + n], z = zp[(size_t)gi * N + n];
            if (s < 1 || s > 127) s = 1;
            if (z > 15) z = 0;
            int u = u4[(size_t)k * N + n];
            const int v = s * (u - z);
            if (u > 15 || v < -128 || v > 127) {
                ++bad;
                u = z;
            }
            size_t cell = ((size_t)(n / 16) * ksteps + k / 128) * 64 + (size_t)((k % 128) / 32) * 16 + n % 16;
            size_t byte = cell * 16 + k % 16;
            if (k % 32 < 16)
                qweight[byte] |= (uint8_t)u;
            else
                qweight[byte] |= (uint8_t)(u << 4);
        }
    }
    return bad;
}

/* Inverse of dgq_oracle_pack_zp. */
void dgq_oracle_unpack_zp(const uint8_t *qweight, const uint8_t *scales_zp, int K, int N, int g,
                          uint8_t *u4, uint8_t *s2, uint8_t *zp)
{
    const int ng = K / g;
    const int gh = (ng + 1) / 2;
    const int ksteps = K / 128;
    for (int gi = 0; gi < ng; ++gi)
        for (int n = 0; n < N; ++n) {
            const size_t at = ((size_t)(n / 16) * gh + gi / 2) * 64 + (size_t)(n % 16) * 4 + (size_t)(gi % 2) * 2;
            s2[(size_t)gi * N + n] = scales_zp[at];
            zp[(size_t)gi * N + n] = scales_zp[at + 1];
        }
    for (int k = 0; k < K; ++k) {
        for (int n = 0; n < N; ++n) {
            size_t cell = ((size_t)(n / 16) * ksteps + k / 128) * 64 + (size_t)((k % 128) / 32) * 16 + n % 16;
            uint8_t b = qweight[cell * 16 + k % 16];
            u4[(size_t)k * N + n] = (uint8_t)((k % 32 < 16) ? (b & 15u) : (b >> 4));
        }
    }
}

/*
 * Static tensor-wise activation quantizer (the "S" scheme of Section 4.1 and Table 5): one
 * scale s for the whole tensor, fixed offline, symmetric form of Eq. 1 with 8 bits:
 *     xq = clamp(round(x / s), -127, 127)          one IEEE division per element, ties to even
 * Values beyond 127 * s saturate (with a dynamic scale they cannot occur).  s must be positive.
 */
void dgq_oracle_quant_act_static(const float *x, long count, float s, int8_t *xq)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < count; ++i) {
        float q = rintf(x[i] / s);
        q = clampf(q, -127.0f, 127.0f);
        xq[i] = (int8_t)q;
    }
}

/*
 * Percentile clipping smoothing (Section 3.4, Eq. 6), offline:
 *     z_j = max_m |X[m][j]|                                   absolute maximum of input channel j
 *     t   = the r-th largest of z, r = ceil(pct * K)          the "top pct" threshold, nearest rank
 *     k_j = max(z_j / t, 1)                                   clamp(., low = 1)
 * so the fewer than r channels above the threshold get k_j > 1 and every other channel 1.
 * If t is zero (no activations), every k_j is 1.  X is [M][K] fp32; k is [K].
 * The scale is then moved from the activations to the weights: X' = X / k, W' = diag(k) W.
 */
static int cmp_desc(const void *a, const void *b)
{
    const float x = *(const float *)a, y = *(const float *)b;
    return x < y ? 1 : (x > y ? -1 : 0);
}

void dgq_oracle_smooth_scales(const float *X, int M, int K, float pct, float *k)
{
    float *z = (float *)malloc(sizeof(float) * (size_t)K);
    float *sorted = (float *)malloc(sizeof(float) * (size_t)K);
    for (int j = 0; j < K; ++j) {
        float a = 0.0f;
        for (int m = 0; m < M; ++m) {
            const float v = fabsf(X[(size_t)m * K + j]);
            if (v > a) a = v;
        }
        z[j] = sorted[j] = a;
    }
    qsort(sorted, (size_t)K, sizeof(float), cmp_desc);
    int r = (int)ceilf(pct * (float)K);
    if (r < 1) r = 1;
    if (r > K) r = K;
    const float t = sorted[r - 1];
    for (int j = 0; j < K; ++j) {
        const float q = t > 0.0f ? z[j] / t : 1.0f;
        k[j] = q < 1.0f ? 1.0f : q;
    }
    free(z);
    free(sorted);
}

/* W'[j][n] = k_j * W[j][n] and X'[m][j] = X[m][j] / k_j in fp32 (the caller rounds to fp16). */
void dgq_oracle_smooth_apply(const float *W, const float *X, const float *k, int M, int K, int N,
                             float *Wout, float *Xout)
{
    for (int j = 0; j < K; ++j)
        for (int n = 0; n < N; ++n) Wout[(size_t)j * N + n] = k[j] * W[(size_t)j * N + n];
    for (int m = 0; m < M; ++m)
        for (int j = 0; j < K; ++j) Xout[(size_t)m * K + j] = X[(size_t)m * K + j] / k[j];
}

/*
 * Producer of the MLP's second linear layer fused with its activation quantizer (the fusion the
 * paper's remark on per-token statistics, Section 4.2, asks for; LLaMA's gated MLP):
 *     h[m][i] = fp16( float( silu(g) * u ) ),  g = GU[m][i], u = GU[m][I + i],
 *     silu(g) = g / (1 + exp(-g))
 * with silu and the product evaluated in fp64, rounded once to fp32 and once more to fp16 (the
 * tensor a model would store), followed by the per-token quantizer of dgq_oracle_quant_act on h.
 * This function writes h as fp32 values that are exactly representable in fp16; the caller
 * quantizes them.  GU is [M][2*I]: the gate columns first, then the up columns.
 */
static float round_to_half(float v)
{
    /* fp32 -> fp16 -> fp32, round to nearest even, by integer arithmetic on the bit pattern */
    union { float f; uint32_t u; } in = {v};
    const uint32_t sign = in.u & 0x80000000u;
    uint32_t x = in.u & 0x7FFFFFFFu;
    union { float f; uint32_t u; } out;
    if (x >= 0x7F800000u) {               /* inf / nan */
        out.u = in.u;
        return out.f;
    }
    if (x >= 0x477FF000u) {               /* rounds to >= 65520: infinity in fp16 */
        out.u = sign | 0x7F800000u;
        return out.f;
    }
    if (x < 0x38800000u) {                /* below 2^-14: fp16 subnormal, spacing 2^-24 */
        const float mag = in.f < 0 ? -in.f : in.f;
        const float q = rintf(mag * 16777216.0f) / 16777216.0f;
        out.f = q;
        out.u |= sign;
        return out.f;
    }
    const uint32_t rem = x & 0x1FFFu;     /* 13 bits dropped */
    x &= ~0x1FFFu;
    if (rem > 0x1000u || (rem == 0x1000u && (x & 0x2000u))) x += 0x2000u;
    out.u = sign | x;
    return out.f;
}

void dgq_oracle_silu_mul(const float *GU, int M, int I, float *h)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int i = 0; i < I; ++i) {
            const double g = (double)GU[(size_t)m * 2 * I + i];
            const double u = (double)GU[(size_t)m * 2 * I + I + i];
            const double p = (g / (1.0 + exp(-g))) * u;
            h[(size_t)m * I + i] = round_to_half((float)p);
        }
    }
}

/*
 * RMSNorm fused with the per-token quantizer (producer of the qkv and gate+up linears of a LLaMA
 * block; same motive as dgq_oracle_silu_mul):
 *     y[m][k] = fp16( float( x * (1 / sqrt(mean_k x^2 + eps)) * gamma[k] ) )
 * with the mean of squares, the reciprocal square root and both products in fp64 (the mean summed
 * in increasing k), rounded once to fp32 and once to fp16; the caller quantizes y per token.
 */
void dgq_oracle_rmsnorm(const float *x, const float *gamma, int M, int K, float eps, float *y)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        double ss = 0.0;
        for (int k = 0; k < K; ++k) ss += (double)x[(size_t)m * K + k] * (double)x[(size_t)m * K + k];
        const double r = 1.0 / sqrt(ss / (double)K + (double)eps);
        for (int k = 0; k < K; ++k)
            y[(size_t)m * K + k] = round_to_half((float)((double)x[(size_t)m * K + k] * r * (double)gamma[k]));
    }
}
