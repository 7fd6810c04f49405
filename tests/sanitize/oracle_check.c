/* Sanitizer driver of the CPU oracle: calls every exported routine of oracle/qii_oracle.c on small
 * ragged shapes, with exactly sized heap buffers, so that AddressSanitizer and
 * UndefinedBehaviorSanitizer see every access and every shift, conversion and index computation.
 * Built and run by tests/test_sanitizers.py:
 *   gcc -O1 -g -std=c11 -fsanitize=address,undefined -fno-sanitize-recover=all -ffp-contract=off
 *       tests/sanitize/oracle_check.c oracle/qii_oracle.c -lm
 * Prints "oracle sanitize: ok" and returns 0 when nothing was reported. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void qo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
void qo_rht_signs(uint64_t seed_rht, uint32_t signbits[4]);
uint32_t qo_scale_draw(uint64_t seed_sr, int64_t row, int64_t cg);
uint32_t qo_elem_draw(uint64_t seed_sr, int64_t row, int64_t col);
uint64_t qo_derive_seed(uint64_t seed, uint32_t i);
float qo_e2m1_decode(uint8_t code);
uint8_t qo_e2m1_rtn(float q);
uint8_t qo_e2m1_sr(float q, uint32_t r16);
float qo_e4m3_decode(uint8_t b);
uint8_t qo_e4m3_rtn(float r);
uint8_t qo_e4m3_sr(float t, uint32_t r20);
float qo_e8m3_rtn(float u);
int qo_rht(const void *x, int dtype, int64_t rows, int64_t cols, int64_t ld, int transpose,
           int rht_group, uint64_t seed_rht, float *y, float *amax);
int qo_quantize(const void *x, int dtype, int64_t rows, int64_t cols, int64_t ld, int transpose,
                int mode, int rht_group, uint64_t seed_rht, uint64_t seed_sr, const float *amax_in,
                float s_override, uint8_t *codes, uint8_t *scales, float *tensor_scale);
int qo_dequantize(const uint8_t *codes, const uint8_t *scales, const float *tensor_scale,
                  int64_t rows, int64_t cols, float *y);
int qo_requantize(const uint8_t *in_codes, const uint8_t *in_scales, const float *in_tensor_scale,
                  int64_t rows, int64_t cols, int transpose, int mode, int rht_group,
                  uint64_t seed_rht, uint64_t seed_sr, const float *amax_in, uint8_t *codes,
                  uint8_t *scales, float *tensor_scale);
int qo_gemm(const uint8_t *a_codes, const uint8_t *a_scales, const float *a_ts, int64_t M,
            const uint8_t *b_codes, const uint8_t *b_scales, const float *b_ts, int64_t N,
            int64_t K, double *C, double *abs_sum);
int qo_gemm_sampled(const uint8_t *a_codes, const uint8_t *a_scales, const float *a_ts,
                    const uint8_t *b_codes, const uint8_t *b_scales, const float *b_ts, int64_t K,
                    const int64_t *ms, const int64_t *ns, int64_t count, double *out, double *abs_sum);
int qo_max_threads(void);

static uint32_t lcg(uint32_t *s) { return *s = *s * 1664525u + 1013904223u; }

/* values over many binades, with zeros, tiny and huge entries */
static float sample(uint32_t *s, int i)
{
    const uint32_t r = lcg(s);
    if (i % 97 == 0) return 0.0f;
    if (i % 211 == 0) return ldexpf(1.0f, 100);
    if (i % 223 == 0) return -ldexpf(1.0f, -120);
    const float m = (float)((r >> 8) & 0xFFFF) / 65536.0f - 0.5f;
    return ldexpf(m, (int)(r & 15) - 8);
}

static int check_shape(int dtype, int64_t rows, int64_t cols, int64_t ld, int transpose, int rht_group)
{
    uint32_t seed = (uint32_t)(rows * 131 + cols * 7 + transpose);
    const size_t n = (size_t)((rows - 1) * ld + cols);   /* exactly the elements the routines may touch */
    const int64_t R = transpose ? cols : rows, C = transpose ? rows : cols;
    void *x;
    if (dtype == 0) {
        float *p = malloc(n * sizeof(float));
        for (size_t i = 0; i < n; ++i) p[i] = sample(&seed, (int)i);
        x = p;
    } else {
        uint16_t *p = malloc(n * sizeof(uint16_t));
        for (size_t i = 0; i < n; ++i) {
            float f = sample(&seed, (int)i);
            uint32_t u;
            memcpy(&u, &f, 4);
            p[i] = (uint16_t)(u >> 16);
        }
        x = p;
    }
    float *y = malloc((size_t)(R * C) * sizeof(float));
    float amax = 0.0f;
    int bad = 0;
    bad |= qo_rht(x, dtype, rows, cols, ld, transpose, rht_group, 5, y, &amax) != 0;
    bad |= qo_rht(x, dtype, rows, cols, ld, transpose, rht_group, 5, y, NULL) != 0;
    uint8_t *codes = malloc((size_t)(R * C / 2)), *scales = malloc((size_t)(R * C / 16));
    uint8_t *codes2 = malloc((size_t)(R * C / 2)), *scales2 = malloc((size_t)(R * C / 16));
    float *deq = malloc((size_t)(R * C) * sizeof(float));
    for (int mode = 0; mode < 5; ++mode) {
        float ts = 0.0f, ts2 = 0.0f;
        bad |= qo_quantize(x, dtype, rows, cols, ld, transpose, mode, rht_group, 5, 9, NULL, 0.0f, codes, scales, &ts) != 0;
        bad |= qo_quantize(x, dtype, rows, cols, ld, transpose, mode, rht_group, 5, 9, &amax, mode == 2 ? 5.5f : 0.0f, codes2, scales2, &ts2) != 0;
        bad |= qo_dequantize(codes, scales, &ts, R, C, deq) != 0;
        /* re-quantization of the saved tensor, plain and transposed (the transposed one needs R % 16 == 0
         * and, with rotation, R % 128 == 0) */
        bad |= qo_requantize(codes, scales, &ts, R, C, 0, mode, rht_group, 6, 10, NULL, codes2, scales2, &ts2) != 0;
        if (R % 16 == 0 && (rht_group == 0 || R % rht_group == 0)) {
            uint8_t *ct = malloc((size_t)(R * C / 2)), *st = malloc((size_t)(R * C / 16));
            bad |= qo_requantize(codes, scales, &ts, R, C, 1, mode, rht_group, 6, 10, NULL, ct, st, &ts2) != 0;
            free(ct);
            free(st);
        }
    }
    /* GEMM of the quantized tensor with itself: M = N = R, K = C */
    {
        float ts = 0.0f;
        qo_quantize(x, dtype, rows, cols, ld, transpose, 0, rht_group, 5, 9, NULL, 0.0f, codes, scales, &ts);
        const int64_t M = R < 5 ? R : 5;
        double *Cm = malloc((size_t)(M * R) * sizeof(double)), *Am = malloc((size_t)(M * R) * sizeof(double));
        bad |= qo_gemm(codes, scales, &ts, M, codes, scales, &ts, R, C, Cm, Am) != 0;
        bad |= qo_gemm(codes, scales, &ts, M, codes, scales, &ts, R, C, Cm, NULL) != 0;
        int64_t ms[3] = {0, M - 1, M / 2}, ns[3] = {R - 1, 0, R / 2};
        double out[3], ab[3];
        bad |= qo_gemm_sampled(codes, scales, &ts, codes, scales, &ts, C, ms, ns, 3, out, ab) != 0;
        bad |= qo_gemm_sampled(codes, scales, &ts, codes, scales, &ts, C, ms, ns, 3, out, NULL) != 0;
        for (int i = 0; i < 3; ++i) bad |= out[i] != Cm[ms[i] * R + ns[i]];
        free(Cm);
        free(Am);
    }
    free(x); free(y); free(codes); free(scales); free(codes2); free(scales2); free(deq);
    if (bad) fprintf(stderr, "oracle sanitize: a call failed for dtype %d %lldx%lld ld %lld transpose %d group %d\n", dtype,
                     (long long)rows, (long long)cols, (long long)ld, transpose, rht_group);
    return bad;
}

int main(void)
{
    int bad = 0;
    /* scalar routines over their whole input ranges */
    uint32_t ctr[4] = {1, 2, 3, 4}, key[2] = {5, 6}, out[4], sg[4];
    qo_philox4x32_10(ctr, key, out);
    qo_rht_signs(0xFFFFFFFFFFFFFFFFull, sg);
    volatile uint32_t sink = qo_scale_draw(~0ull, INT64_MAX / 4, INT64_MAX / 4) ^ qo_elem_draw(~0ull, INT64_MAX / 4, 3);
    sink ^= (uint32_t)qo_derive_seed(~0ull, 5);
    for (int c = 0; c < 256; ++c) {
        sink ^= (uint32_t)qo_e2m1_decode((uint8_t)c);
        sink ^= (uint32_t)qo_e4m3_decode((uint8_t)c);
    }
    const float probes[] = {0.0f, -0.0f, 1e-45f, 1e-30f, 0.24f, 0.25f, 0.75f, 1.25f, 5.0f, 6.0f, 7.0f, 447.0f, 448.0f, 449.0f,
                            1e30f, 3.4e38f, -3.4e38f, -1e-45f, 0.001953125f, 0.0009765625f, 240.0f, 256.0f, 464.0f};
    for (size_t i = 0; i < sizeof probes / sizeof probes[0]; ++i) {
        sink ^= qo_e2m1_rtn(probes[i]);
        sink ^= qo_e2m1_sr(probes[i], 0u) ^ qo_e2m1_sr(probes[i], 0xFFFFu);
        sink ^= qo_e4m3_rtn(fabsf(probes[i]));
        sink ^= qo_e4m3_sr(fabsf(probes[i]) > 448.0f ? 448.0f : fabsf(probes[i]), 0u) ^ qo_e4m3_sr(fabsf(probes[i]) > 448.0f ? 448.0f : fabsf(probes[i]), 0xFFFFFu);
        sink ^= (uint32_t)qo_e8m3_rtn(fabsf(probes[i]));
    }
    sink ^= (uint32_t)qo_max_threads();
    /* tensor routines: smallest, ragged and padded shapes, both dtypes, both orientations */
    bad |= check_shape(0, 1, 16, 16, 0, 0);
    bad |= check_shape(1, 1, 128, 128, 0, 128);
    bad |= check_shape(0, 3, 48, 50, 0, 0);
    bad |= check_shape(1, 5, 256, 260, 0, 128);
    bad |= check_shape(0, 16, 7, 9, 1, 0);
    bad |= check_shape(1, 128, 3, 3, 1, 128);
    bad |= check_shape(0, 256, 32, 40, 1, 128);
    bad |= check_shape(1, 128, 128, 128, 0, 128);
    bad |= check_shape(1, 128, 128, 136, 1, 128);
    /* rejected shapes return an error and touch nothing */
    {
        float xx[8] = {0}, ts;
        uint8_t b[8];
        bad |= qo_quantize(xx, 0, 1, 8, 8, 0, 0, 0, 1, 2, NULL, 0.0f, b, b, &ts) == 0;
        bad |= qo_quantize(xx, 0, 1, 16, 16, 0, 7, 0, 1, 2, NULL, 0.0f, b, b, &ts) == 0;
        bad |= qo_dequantize(b, b, &ts, 1, 8, xx) == 0;
    }
    if (bad) return 1;
    printf("oracle sanitize: ok (%u)\n", (unsigned)(sink & 1u));
    return 0;
}
