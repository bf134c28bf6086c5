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
 * numpy int64 matmul, an fp64 group-wise "segmented GEMM").  The statistical
 * accuracy of the RTN quantizer against the paper's perplexity tables is
 * parity unpinned (needs the trained models and datasets).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
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
