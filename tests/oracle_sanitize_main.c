/* Driver for tests/test_oracle_sanitized.py: runs every oracle function once on small inputs with
 * exactly sized heap buffers, so that AddressSanitizer / UndefinedBehaviorSanitizer see any access
 * past a buffer, signed overflow or bad shift in the oracle's index arithmetic.  Prints "ok". */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void dgq_oracle_quantize_rtn(const float *, int, int, int, int8_t *, uint8_t *, float *);
void dgq_oracle_quant_act(const float *, int, int, int8_t *, float *);
long dgq_oracle_expand(const int8_t *, const uint8_t *, int, int, int, int8_t *);
long dgq_oracle_gemm_i32(const int8_t *, const int8_t *, int, int, int, int32_t *);
void dgq_oracle_epilogue(const int32_t *, const float *, const float *, int, int, float *);
long dgq_oracle_pack(const int8_t *, const uint8_t *, int, int, int, uint8_t *, uint8_t *);
void dgq_oracle_unpack(const uint8_t *, const uint8_t *, int, int, int, int8_t *, uint8_t *);
long dgq_oracle_expand_zp(const uint8_t *, const uint8_t *, const uint8_t *, int, int, int, int8_t *);
void dgq_oracle_quantize_grid(const float *, int, int, int, int, float, uint8_t *, uint8_t *, uint8_t *, float *);
long dgq_oracle_pack_zp(const uint8_t *, const uint8_t *, const uint8_t *, int, int, int, uint8_t *, uint8_t *);
void dgq_oracle_unpack_zp(const uint8_t *, const uint8_t *, int, int, int, uint8_t *, uint8_t *, uint8_t *);
void dgq_oracle_quant_act_static(const float *, long, float, int8_t *);

static unsigned long long st = 88172645463325252ull;
static float rnd(void)
{
    st ^= st << 13, st ^= st >> 7, st ^= st << 17;
    return (float)((double)(st % 20001) / 10000.0 - 1.0);
}

int main(void)
{
    /* ragged on purpose: three groups (padding in both scale layouts), 48 columns */
    const int M = 5, K = 384, N = 48, g = 128, ng = K / g;
    float *W = malloc(sizeof(float) * K * N), *x = malloc(sizeof(float) * M * K);
    for (int i = 0; i < K * N; ++i) W[i] = 0.02f * rnd();
    for (int i = 0; i < M * K; ++i) x[i] = rnd();
    int8_t *w4 = malloc(K * N), *ws8 = malloc(K * N), *xq = malloc(M * K), *w4b = malloc(K * N);
    uint8_t *s2 = malloc(ng * N), *s2b = malloc(ng * N), *zp = malloc(ng * N), *zpb = malloc(ng * N);
    uint8_t *u4 = malloc(K * N), *u4b = malloc(K * N);
    float *s1 = malloc(sizeof(float) * N), *sx = malloc(sizeof(float) * M), *out = malloc(sizeof(float) * M * N);
    int32_t *acc = malloc(sizeof(int32_t) * M * N);
    uint8_t *qw = malloc((size_t)K * N / 2), *sc = malloc((size_t)(N / 16) * ((ng + 3) / 4) * 64);
    uint8_t *scz = malloc((size_t)(N / 16) * ((ng + 1) / 2) * 64);
    long bad = 0;

    dgq_oracle_quantize_rtn(W, K, N, g, w4, s2, s1);
    dgq_oracle_quant_act(x, M, K, xq, sx);
    bad += dgq_oracle_expand(w4, s2, K, N, g, ws8);
    bad += dgq_oracle_gemm_i32(xq, ws8, M, N, K, acc);
    dgq_oracle_epilogue(acc, sx, s1, M, N, out);
    bad += dgq_oracle_pack(w4, s2, K, N, g, qw, sc);
    dgq_oracle_unpack(qw, sc, K, N, g, w4b, s2b);
    for (int i = 0; i < K * N; ++i) bad += w4[i] != w4b[i];

    dgq_oracle_quantize_grid(W, K, N, g, 11, 0.05f, u4, zp, s2, s1);
    bad += dgq_oracle_expand_zp(u4, s2, zp, K, N, g, ws8);
    bad += dgq_oracle_pack_zp(u4, s2, zp, K, N, g, qw, scz);
    dgq_oracle_unpack_zp(qw, scz, K, N, g, u4b, s2b, zpb);
    for (int i = 0; i < K * N; ++i) bad += u4[i] != u4b[i];
    for (int i = 0; i < ng * N; ++i) bad += (s2[i] != s2b[i]) + (zp[i] != zpb[i]);
    dgq_oracle_quant_act_static(x, (long)M * K, 0.01f, xq);

    printf(bad ? "mismatch %ld\n" : "ok\n", bad);
    free(W), free(x), free(w4), free(ws8), free(xq), free(w4b), free(s2), free(s2b), free(zp), free(zpb);
    free(u4), free(u4b), free(s1), free(sx), free(out), free(acc), free(qw), free(sc), free(scz);
    return bad != 0;
}
