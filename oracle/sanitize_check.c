/*
 * sanitize_check.c -- TEST INFRASTRUCTURE ONLY: a small driver that runs every entry point of the fp64
 * oracle (naut_oracle.c) and of the input generator (naut_synth.c) on tiny, awkward shapes, meant to be
 * compiled together with both sources under -fsanitize=address,undefined (tests/test_sanitize.py does
 * that and runs it): an out-of-bounds index, a misaligned or overflowing computation in the host code
 * aborts it with a sanitizer report.  It checks no values beyond finiteness and two closed forms (V = 1
 * gives O = 1; one key gives lse = its score); the pins of the oracle live in tests/test_oracle_pins.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int naut_oracle_attn_f64(const double *q, const double *k, const double *v, double *o, double *lse, double *probs,
                         int B, int Hq, int Hkv, int S, int D, int causal, double scale);
int naut_oracle_attn_rows(const uint16_t *q, const uint16_t *k, const uint16_t *v, int in_dtype, const int64_t *rows,
                          int64_t nrows, double *o, double *lse, int B, int Hq, int Hkv, int S, int D, int causal,
                          double scale);
int naut_oracle_attn_cross_f64(const double *q, const double *k, const double *v, double *o, double *lse, int B, int Hq,
                               int Hkv, int Sq, int Sk, int D, int causal, double scale);
int naut_oracle_attn_cross16(const uint16_t *q, const uint16_t *k, const uint16_t *v, int in_dtype, double *o,
                             double *lse, int B, int Hq, int Hkv, int Sq, int Sk, int D, int causal, double scale);
int naut_oracle_decode_e4m3(const uint8_t *bits, double *out, int64_t n);
int naut_oracle_attn_rows_e4m3(const uint8_t *q, const uint8_t *k, const uint8_t *v, double dq, double dk, double dv,
                               const int64_t *rows, int64_t nrows, double *o, double *lse, int B, int Hq, int Hkv,
                               int S, int D, int causal, double scale);
int naut_oracle_decode16(const uint16_t *bits, int dtype, double *out, int64_t n);
int naut_oracle_threads(void);
int naut_synth_fill(uint16_t *out, int B, int H, int S, int D, uint64_t seed, uint32_t tag, int dtype, int n_outlier,
                    float outlier_scale);
int naut_synth_outlier_rows(int32_t *rows, int64_t bh, int S, uint64_t seed, uint32_t tag, int n_outlier);
int naut_synth_round16(const float *in, uint16_t *out, int64_t n, int dtype);
int naut_synth_round_e4m3(const float *in, uint8_t *out, int64_t n);

static int failures = 0;
#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            fprintf(stderr, "sanitize_check: %s failed (line %d)\n", #cond, __LINE__); \
            ++failures;                                                    \
        }                                                                  \
    } while (0)

static int all_finite(const double *x, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        if (!isfinite(x[i]))
            return 0;
    return 1;
}

static void one_shape(int B, int Hq, int Hkv, int S, int D, int causal, int dtype)
{
    const size_t nq = (size_t)B * Hq * S * D, nk = (size_t)B * Hkv * S * D, nr = (size_t)B * Hq * S;
    uint16_t *q = malloc(nq * 2), *k = malloc(nk * 2), *v = malloc(nk * 2);
    double *o = malloc(nq * 8), *lse = malloc(nr * 8);
    const int n_out = S / 3;
    CHECK(naut_synth_fill(q, B, Hq, S, D, 77, 1, dtype, 0, 1.0f) == 0);
    CHECK(naut_synth_fill(k, B, Hkv, S, D, 77, 2, dtype, n_out, 8.0f) == 0);
    CHECK(naut_synth_fill(v, B, Hkv, S, D, 77, 3, dtype, 0, 1.0f) == 0);
    const double scale = 1.0 / sqrt((double)D);
    /* all rows, then a subset given by index (first, last, one in between, out of order) */
    CHECK(naut_oracle_attn_rows(q, k, v, dtype, NULL, (int64_t)nr, o, lse, B, Hq, Hkv, S, D, causal, scale) == 0);
    CHECK(all_finite(o, nq) && all_finite(lse, nr));
    int64_t rows[3] = {(int64_t)nr - 1, 0, (int64_t)nr / 2};
    double *o3 = malloc(3 * (size_t)D * 8), lse3[3];
    CHECK(naut_oracle_attn_rows(q, k, v, dtype, rows, 3, o3, lse3, B, Hq, Hkv, S, D, causal, scale) == 0);
    for (int r = 0; r < 3; ++r)
        CHECK(memcmp(o3 + (size_t)r * D, o + (size_t)rows[r] * D, (size_t)D * 8) == 0 && lse3[r] == lse[rows[r]]);
    /* the same inputs through the fp64 entry (with the probability matrix) and the cross entries */
    double *qd = malloc(nq * 8), *kd = malloc(nk * 8), *vd = malloc(nk * 8), *o2 = malloc(nq * 8), *lse2 = malloc(nr * 8);
    double *probs = malloc(nr * (size_t)S * 8);
    CHECK(naut_oracle_decode16(q, dtype, qd, (int64_t)nq) == 0);
    CHECK(naut_oracle_decode16(k, dtype, kd, (int64_t)nk) == 0);
    CHECK(naut_oracle_decode16(v, dtype, vd, (int64_t)nk) == 0);
    CHECK(naut_oracle_attn_f64(qd, kd, vd, o2, lse2, probs, B, Hq, Hkv, S, D, causal, scale) == 0);
    CHECK(memcmp(o, o2, nq * 8) == 0);
    CHECK(naut_oracle_attn_cross_f64(qd, kd, vd, o2, lse2, B, Hq, Hkv, S, S, D, causal, scale) == 0);
    CHECK(all_finite(o2, nq));
    CHECK(naut_oracle_attn_cross16(q, k, v, dtype, o2, lse2, B, Hq, Hkv, S, S, D, causal, scale) == 0);
    CHECK(all_finite(o2, nq));
    /* V = 1 gives O = 1 */
    for (size_t i = 0; i < nk; ++i)
        vd[i] = 1.0;
    CHECK(naut_oracle_attn_f64(qd, kd, vd, o2, NULL, NULL, B, Hq, Hkv, S, D, causal, scale) == 0);
    for (size_t i = 0; i < nq; ++i)
        CHECK(fabs(o2[i] - 1.0) < 1e-12);
    int32_t *orow = malloc((size_t)(n_out > 0 ? n_out : 1) * 4);
    CHECK(naut_synth_outlier_rows(orow, 0, S, 77, 2, n_out) == 0);
    for (int i = 0; i < n_out; ++i)
        CHECK(orow[i] >= 0 && orow[i] < S);
    free(q); free(k); free(v); free(o); free(lse); free(o3); free(qd); free(kd); free(vd); free(o2); free(lse2);
    free(probs); free(orow);
}

static void fp8_shape(int B, int Hq, int Hkv, int S, int D, int causal)
{
    const size_t nq = (size_t)B * Hq * S * D, nk = (size_t)B * Hkv * S * D, nr = (size_t)B * Hq * S;
    float *f = malloc((nq > nk ? nq : nk) * 4);
    uint8_t *q = malloc(nq), *k = malloc(nk), *v = malloc(nk);
    for (size_t i = 0; i < nq; ++i)
        f[i] = (float)((int)(i * 2654435761u % 2001) - 1000) * 0.5f;   /* -500 .. 500: saturation and subnormals */
    CHECK(naut_synth_round_e4m3(f, q, (int64_t)nq) == 0);
    for (size_t i = 0; i < nk; ++i)
        f[i] = (float)((int)(i * 40503u % 257) - 128) * 0.01f;
    CHECK(naut_synth_round_e4m3(f, k, (int64_t)nk) == 0);
    CHECK(naut_synth_round_e4m3(f, v, (int64_t)nk) == 0);
    double *o = malloc(nq * 8), *lse = malloc(nr * 8), dec[256];
    uint8_t codes[256];
    for (int i = 0; i < 256; ++i)
        codes[i] = (uint8_t)i;
    CHECK(naut_oracle_decode_e4m3(codes, dec, 256) == 0);
    CHECK(naut_oracle_attn_rows_e4m3(q, k, v, 1.0 / 64, 0.125, 1.0 / 64, NULL, (int64_t)nr, o, lse, B, Hq, Hkv, S, D, causal,
                                     1.0 / sqrt((double)D)) == 0);
    CHECK(all_finite(o, nq) && all_finite(lse, nr));
    free(f); free(q); free(k); free(v); free(o); free(lse);
}

int main(void)
{
    CHECK(naut_oracle_threads() >= 1);
    one_shape(1, 1, 1, 1, 8, 0, 0);      /* a single key: lse = its score */
    one_shape(1, 1, 1, 1, 8, 1, 1);
    one_shape(2, 4, 2, 37, 24, 1, 0);    /* grouped heads, odd sizes, causal */
    one_shape(1, 3, 1, 65, 64, 0, 1);    /* fp16, non-causal */
    one_shape(3, 2, 2, 5, 128, 1, 0);
    fp8_shape(1, 2, 1, 19, 16, 1);
    fp8_shape(2, 2, 2, 33, 64, 0);
    /* bad arguments are reported, not dereferenced */
    double d1[8];
    uint16_t u1[8] = {0};
    CHECK(naut_oracle_attn_rows(NULL, u1, u1, 0, NULL, 1, d1, NULL, 1, 1, 1, 1, 8, 0, 1.0) == -1);
    CHECK(naut_oracle_attn_rows(u1, u1, u1, 0, NULL, 1, d1, NULL, 1, 3, 2, 1, 8, 0, 1.0) == -1);
    CHECK(naut_synth_fill(u1, 1, 1, 1, 8, 1, 1, 0, 2, 1.0f) == -1);
    /* rounding entry on the edges of both 16-bit formats */
    const float edge[8] = {0.0f, -0.0f, 1.0f, 65504.0f, 65520.0f, 1e-8f, -3.3895314e38f, 5.9604645e-8f};
    CHECK(naut_synth_round16(edge, u1, 8, 0) == 0);
    CHECK(naut_synth_round16(edge, u1, 8, 1) == 0);
    if (failures) {
        fprintf(stderr, "sanitize_check: %d check(s) failed\n", failures);
        return 1;
    }
    printf("sanitize_check: ok\n");
    return 0;
}
