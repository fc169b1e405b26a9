/* Driver of the CPU oracle for a build under -fsanitize=address,undefined (run by
 * tests/test_sanitizers.py).  It walks every oracle entry point over small shapes that include
 * the extremes of the code ranges at the longest reduction the interface admits, so that a
 * signed overflow, an out-of-range shift or an access beyond a buffer aborts the run.
 * Prints "ok" and exits 0 when nothing trapped. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_choose_qparams(double, double, int, float *, int32_t *);
int oracle_act_range(int, float, int32_t, int32_t *, int32_t *);
int oracle_quantize(const float *, uint8_t *, size_t, float, int32_t, int32_t, int32_t);
int oracle_dequantize(const uint8_t *, float *, size_t, float, int32_t);
int oracle_quantize_wide(const float *, uint16_t *, size_t, float, int32_t, int32_t, int32_t);
int oracle_dequantize_wide(const uint16_t *, float *, size_t, float, int32_t);
int oracle_quantize_weights(const float *, size_t, size_t, int, int, int8_t *, float *);
int oracle_pack_int4(const int8_t *, size_t, uint8_t *);
int oracle_unpack_int4(const uint8_t *, size_t, int8_t *);
int oracle_quantize_multiplier(double, int32_t *, int32_t *);
int32_t oracle_rescale(int32_t, int32_t, int32_t);
int oracle_requantize(const int32_t *, uint8_t *, size_t, size_t, const int32_t *, const int32_t *, int, int32_t, int32_t,
                      int32_t);
int oracle_qgemm(const uint8_t *, int64_t, int32_t, const void *, int64_t, int, const int32_t *, int64_t, int64_t, int64_t,
                 const int32_t *, const int32_t *, const int32_t *, int32_t, int32_t, int32_t, uint8_t *, int64_t);
int oracle_qconv2d(const uint8_t *, int, int, int, int, int32_t, const void *, int, int, int, int, const int32_t *, int, int,
                   int, int, const int32_t *, const int32_t *, const int32_t *, int32_t, int32_t, int32_t, uint8_t *,
                   const int64_t *, int64_t);
int oracle_qdwconv2d(const uint8_t *, int, int, int, int, int32_t, const int8_t *, int, int, const int32_t *, int, int, int,
                     int, const int32_t *, const int32_t *, const int32_t *, int32_t, int32_t, int32_t, uint8_t *,
                     const int64_t *, int64_t);
int oracle_qadd(const uint8_t *, int32_t, int32_t, int32_t, const uint8_t *, int32_t, int32_t, int32_t, int32_t, int32_t,
                int32_t, int32_t, int32_t, int32_t, uint8_t *, size_t);
int oracle_qadd_params(double, double, double, int32_t *, int32_t *, int32_t *, int32_t *, int32_t *, int32_t *, int32_t *);

static uint32_t rng_state = 180608342u;
static uint32_t rnd(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state >> 8;
}

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); \
            return 1;                                                      \
        }                                                                  \
    } while (0)

int main(void)
{
    /* quantizer parameters and the element-wise pair, special values included */
    float s;
    int32_t z, lo, hi;
    CHECK(oracle_choose_qparams(2.1, 3.5, 8, &s, &z) == 0 && z == 0);
    CHECK(oracle_choose_qparams(-1e30, 1e30, 8, &s, &z) == 0);
    CHECK(oracle_choose_qparams(0.0, 0.0, 4, &s, &z) == 0);
    CHECK(oracle_act_range(2, 6.0f / 255, 0, &lo, &hi) == 0 && hi == 255);
    float xs[8] = {0.0f, -0.0f, NAN, INFINITY, -INFINITY, 3.4e38f, -3.4e38f, 1e-45f};
    uint8_t q[8];
    float back[8];
    CHECK(oracle_quantize(xs, q, 8, 1e-6f, 128, 0, 255) == 0);
    CHECK(oracle_dequantize(q, back, 8, 1e-6f, 128) == 0);
    CHECK(q[3] == 255 && q[4] == 0 && q[2] == 128);
    uint16_t qw[8];
    CHECK(oracle_quantize_wide(xs, qw, 8, 1e-6f, 32768, 0, 65535) == 0);
    CHECK(oracle_dequantize_wide(qw, back, 8, 1e-6f, 32768) == 0);
    CHECK(qw[3] == 65535 && qw[4] == 0 && qw[2] == 32768);
    CHECK(oracle_quantize_wide(xs, qw, 8, 1e-6f, 0, 0, 65536) != 0);

    /* weights: 8 and 4 bits, packing */
    float wf[2 * 6] = {-1.0f, 0.5f, 0.25f, 0.0f, 1.0f, -0.125f, 0, 0, 0, 0, 0, 0};
    int8_t wq[12];
    float d[2];
    CHECK(oracle_quantize_weights(wf, 2, 6, 8, 1, wq, d) == 0);
    CHECK(oracle_quantize_weights(wf, 2, 6, 4, 0, wq, d) == 0);
    uint8_t packed[6];
    int8_t unpacked[12];
    CHECK(oracle_pack_int4(wq, 12, packed) == 0 && oracle_unpack_int4(packed, 12, unpacked) == 0);
    CHECK(memcmp(wq, unpacked, 12) == 0);

    /* rescale: every shift the interface admits, extreme accumulators and multipliers */
    const int32_t accs[] = {INT32_MIN, INT32_MIN + 1, -(1 << 30), -1, 0, 1, (1 << 30), INT32_MAX - 1, INT32_MAX};
    const int32_t mults[] = {0, 1, 1 << 30, INT32_MAX, INT32_MIN};
    for (unsigned a = 0; a < sizeof accs / sizeof *accs; ++a)
        for (unsigned m = 0; m < sizeof mults / sizeof *mults; ++m)
            for (int sh = -31; sh <= 31; ++sh) (void)oracle_rescale(accs[a], mults[m], sh);
    int32_t mu, sf;
    CHECK(oracle_quantize_multiplier(1.0 - ldexp(1.0, -40), &mu, &sf) == 0 && mu == (1 << 30) && sf == -1);
    CHECK(oracle_quantize_multiplier(ldexp(1.0, -33), &mu, &sf) == 0);
    int32_t big[6] = {INT32_MIN, INT32_MAX, 0, -1, 1, 12345};
    int32_t pm[3] = {INT32_MAX, 1 << 30, 0}, ps[3] = {-31, 31, 0};
    uint8_t y6[6];
    CHECK(oracle_requantize(big, y6, 2, 3, pm, ps, 1, 255, 0, 255) == 0);

    /* dense product at the longest reduction with the extreme codes: |sum| reaches K * 255 * 128 */
    const int64_t K = 65536, M = 2, N = 3;
    uint8_t *A = malloc((size_t)(M * K));
    int8_t *B = malloc((size_t)(N * K));
    CHECK(A && B);
    for (int64_t k = 0; k < K; ++k) {
        A[k] = 255, A[K + k] = 0;
        B[k] = -128, B[K + k] = 127, B[2 * K + k] = (int8_t)(rnd() & 0xff);
    }
    int32_t bias[3] = {0, 0, 0}, mul3[3] = {1 << 30, 1 << 30, 1 << 30}, sh3[3] = {20, 20, 20};
    uint8_t C[6];
    CHECK(oracle_qgemm(A, K, 0, B, K, 8, NULL, M, N, K, bias, mul3, sh3, 128, 0, 255, C, N) == 0);
    int32_t zw3[3] = {-128, 127, 5};
    /* with weight zero-points the bound on K halves */
    CHECK(oracle_qgemm(A, K, 255, B, K, 8, zw3, M, N, 32768, bias, mul3, sh3, 128, 0, 255, C, N) == 0);
    /* packed 4-bit weights over the same buffer */
    CHECK(oracle_qgemm(A, K, 128, B, 2 * K, 4, NULL, M, 1, 2 * 1024, bias, mul3, sh3, 128, 0, 255, C, 1) == 0);
    free(A), free(B);

    /* convolutions with padding wider than the kernel reach, strides, sampling, weight zero-points */
    enum { NI = 2, H = 5, W = 4, CI = 6, CO = 3 };
    uint8_t x[NI * H * W * CI];
    int8_t w[CO * 3 * 3 * CI], wd[3 * 3 * CI];
    for (unsigned i = 0; i < sizeof x; ++i) x[i] = (uint8_t)rnd();
    for (unsigned i = 0; i < sizeof w; ++i) w[i] = (int8_t)rnd();
    for (unsigned i = 0; i < sizeof wd; ++i) wd[i] = (int8_t)rnd();
    int32_t cb[CI] = {1, -2, 3, -4, 5, -6}, cm[CI], cs[CI], czw[CI] = {-128, 127, 0, 1, -1, 64};
    for (int i = 0; i < CI; ++i) cm[i] = (1 << 30) + i, cs[i] = 8 + i;
    uint8_t yo[NI * 7 * 6 * CI];
    for (int sh = 1; sh <= 2; ++sh)
        for (int pad = 0; pad <= 2; ++pad) {
            CHECK(oracle_qconv2d(x, NI, H, W, CI, 77, w, CO, 3, 3, 8, pad ? czw : NULL, sh, 1, pad, pad, cb, cm, cs, 3, 0, 255,
                                 yo, NULL, 0) == 0);
            CHECK(oracle_qdwconv2d(x, NI, H, W, CI, 77, wd, 3, 3, pad ? czw : NULL, sh, sh, pad, pad, cb, cm, cs, 3, 0, 255, yo,
                                   NULL, 0) == 0);
        }
    int64_t sample[3] = {0, 5, NI * H * W * CO - 1};
    CHECK(oracle_qconv2d(x, NI, H, W, CI, 77, w, CO, 3, 3, 8, NULL, 1, 1, 1, 1, cb, cm, cs, 3, 0, 255, yo, sample, 3) == 0);
    int64_t bad_sample[1] = {(int64_t)NI * H * W * CO};
    CHECK(oracle_qconv2d(x, NI, H, W, CI, 77, w, CO, 3, 3, 8, NULL, 1, 1, 1, 1, cb, cm, cs, 3, 0, 255, yo, bad_sample, 1) != 0);

    /* rescaling add over all code pairs for a few scale triples */
    uint8_t *pa = malloc(65536), *pb = malloc(65536), *py = malloc(65536);
    CHECK(pa && pb && py);
    for (int i = 0; i < 65536; ++i) pa[i] = (uint8_t)(i >> 8), pb[i] = (uint8_t)i;
    const double triples[3][3] = {{0.02, 0.031, 0.04}, {1.0, 1e-3, 0.5}, {1e-4, 1e-4, 1e-2}};
    for (int t = 0; t < 3; ++t) {
        int32_t p[7];
        CHECK(oracle_qadd_params(triples[t][0], triples[t][1], triples[t][2], &p[0], &p[1], &p[2], &p[3], &p[4], &p[5], &p[6]) == 0);
        CHECK(oracle_qadd(pa, 0, p[1], p[2], pb, 255, p[3], p[4], p[0], p[5], p[6], 128, 0, 255, py, 65536) == 0);
    }
    free(pa), free(pb), free(py);
    puts("ok");
    return 0;
}
