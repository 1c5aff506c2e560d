/*
 * naut_oracle.c -- fp64 CPU oracle for softmax attention.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the checker, not the product.  Only the test-suite, the smoke
 * check and the benchmark's cpu_baseline leg may load it.  It shares no code,
 * header, table or helper with the HIP path and is never a fallback for it.
 *
 * What it computes: the operator the paper takes as its math-level input, two matrix
 * products with a softmax between them (Section 1, and the operator table in
 * Section 6: Global, Causal and Grouped-Query attention), i.e. for every batch b, query head h, query i
 *
 *   pass 1 (scores)       s_ij = scale * sum_d q[b,h,i,d] * k[b,hk(h),j,d],   j in J_i
 *   pass 2 (softmax)      m_i = max_j s_ij ; p_ij = exp(s_ij - m_i) ;
 *                         l_i = sum_j p_ij ; P_ij = p_ij / l_i
 *   pass 3 (weighted sum) o[b,h,i,d] = sum_j P_ij * v[b,hk(h),j,d]
 *                         lse[b,h,i] = m_i + ln(l_i)
 *
 * with J_i = {0..S-1} (global) or {0..i} (causal, diagonal included) and
 * hk(h) = floor(h / (Hq/Hkv)) (grouped-query: consecutive query heads share one
 * key/value head).  It is the unfused FP64 reference the paper's numerical
 * study (Appendix B) compares fused kernels against: three separate passes,
 * no tiling, no online rescaling, no exp2 rewrite, no fusion.
 *
 * Layout: q,o [B][Hq][S][D]; k,v [B][Hkv][S][D]; lse [B][Hq][S]; D innermost.
 * All pointers are host memory.  Outputs are fp64.
 *
 * Pinned (tests/test_oracle_pins.py) by: hand-expanded sums at S<=4, rows of P
 * summing to one, V=1 => O=1, Q=0 => prefix/column mean of V and lse=ln|J_i|,
 * key permutation invariance, causal row 0, the prefix property, GQA ==
 * repeated-head MHA, (q,scale)->(2q,scale/2), key-shift, split-merge, the
 * one-hot limit and a SciPy softmax/logsumexp second opinion.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define NAUT_ORACLE_BF16 0
#define NAUT_ORACLE_F16 1

/* ---- exact decoders of 16-bit storage formats to fp64 ------------------- */

/* bfloat16: the upper 16 bits of an IEEE binary32. */
static double decode_bf16(uint16_t bits)
{
    uint32_t w = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
static double decode_f16(uint16_t bits)
{
    int sign = (bits >> 15) & 1;
    int expo = (bits >> 10) & 0x1f;
    int frac = bits & 0x3ff;
    double mag;
    if (expo == 0)
        mag = ldexp((double)frac, -24); /* subnormal: frac * 2^-10 * 2^-14 */
    else if (expo == 31)
        mag = frac ? NAN : INFINITY;
    else
        mag = ldexp(1.0 + (double)frac / 1024.0, expo - 15);
    return sign ? -mag : mag;
}

static double decode16(uint16_t bits, int dtype)
{
    return dtype == NAUT_ORACLE_F16 ? decode_f16(bits) : decode_bf16(bits);
}

/* ---- one query row, three passes ---------------------------------------- */

/*
 * qrow[D]; K, V point at key 0 of the row's key/value head ([S][D]).
 * nkeys = |J_i|.  s[nkeys] is caller scratch; on return it holds P_i (the
 * normalised probabilities).  o[D] and *lse receive the row's outputs.
 */
static void attn_row(const double *qrow, const double *K, const double *V, int64_t nkeys, int D,
                     double scale, double *s, double *o, double *lse)
{
    /* pass 1: scores */
    for (int64_t j = 0; j < nkeys; ++j) {
        double acc = 0.0;
        for (int d = 0; d < D; ++d)
            acc += qrow[d] * K[j * D + d];
        s[j] = scale * acc;
    }
    /* pass 2: explicit softmax */
    double m = s[0];
    for (int64_t j = 1; j < nkeys; ++j)
        if (s[j] > m)
            m = s[j];
    double l = 0.0;
    for (int64_t j = 0; j < nkeys; ++j) {
        s[j] = exp(s[j] - m);
        l += s[j];
    }
    for (int64_t j = 0; j < nkeys; ++j)
        s[j] /= l;
    /* pass 3: weighted sum of value rows */
    for (int d = 0; d < D; ++d)
        o[d] = 0.0;
    for (int64_t j = 0; j < nkeys; ++j)
        for (int d = 0; d < D; ++d)
            o[d] += s[j] * V[j * D + d];
    *lse = m + log(l);
}

static int bad_shape(int B, int Hq, int Hkv, int S, int D)
{
    return B <= 0 || Hq <= 0 || Hkv <= 0 || S <= 0 || D <= 0 || Hq % Hkv != 0;
}

/* ---- fp64-in entry points ------------------------------------------------ */

/*
 * Full attention on fp64 inputs.  o [B][Hq][S][D], lse [B][Hq][S] (may be NULL),
 * probs [B][Hq][S][S] (may be NULL; masked positions are written as 0).
 * Returns 0, or -1 on a bad shape / NULL pointer, -2 if scratch cannot be had.
 */
int naut_oracle_attn_f64(const double *q, const double *k, const double *v, double *o, double *lse,
                         double *probs, int B, int Hq, int Hkv, int S, int D, int causal,
                         double scale)
{
    if (!q || !k || !v || !o || bad_shape(B, Hq, Hkv, S, D))
        return -1;
    const int g = Hq / Hkv;
    const int64_t nrows = (int64_t)B * Hq * S;
    int err = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)S);
        if (!s) {
#pragma omp atomic write
            err = -2;
        }
#pragma omp for schedule(dynamic, 16)
        for (int64_t r = 0; r < nrows; ++r) {
            if (!s)
                continue;
            const int64_t i = r % S;
            const int64_t h = (r / S) % Hq;
            const int64_t b = r / ((int64_t)S * Hq);
            const int64_t hk = h / g;
            const int64_t nkeys = causal ? i + 1 : S;
            const double *Kh = k + (b * Hkv + hk) * (int64_t)S * D;
            const double *Vh = v + (b * Hkv + hk) * (int64_t)S * D;
            double lse_r;
            attn_row(q + r * D, Kh, Vh, nkeys, D, scale, s, o + r * D, &lse_r);
            if (lse)
                lse[r] = lse_r;
            if (probs) {
                for (int64_t j = 0; j < S; ++j)
                    probs[r * S + j] = j < nkeys ? s[j] : 0.0;
            }
        }
        free(s);
    }
    return err;
}

/* ---- 16-bit-in entry points ---------------------------------------------- */

/*
 * Attention for a chosen list of query rows, inputs given as bf16/fp16 bit
 * patterns (decoded exactly).  rows[n] holds linear row ids r = (b*Hq + h)*S + i.
 * rows == NULL means all B*Hq*S rows in order (then nrows must equal B*Hq*S).
 * o [nrows][D], lse [nrows] (may be NULL).  Every output row depends only on its
 * own query row and on K,V[J_i], so any subset is exact.
 * Returns 0, -1 on bad arguments, -2 if memory cannot be had.
 */
int naut_oracle_attn_rows(const uint16_t *q, const uint16_t *k, const uint16_t *v, int in_dtype,
                          const int64_t *rows, int64_t nrows, double *o, double *lse, int B, int Hq,
                          int Hkv, int S, int D, int causal, double scale)
{
    if (!q || !k || !v || !o || bad_shape(B, Hq, Hkv, S, D) || nrows < 0)
        return -1;
    if (in_dtype != NAUT_ORACLE_BF16 && in_dtype != NAUT_ORACLE_F16)
        return -1;
    const int64_t total = (int64_t)B * Hq * S;
    if (!rows && nrows != total)
        return -1;
    if (rows)
        for (int64_t t = 0; t < nrows; ++t)
            if (rows[t] < 0 || rows[t] >= total)
                return -1;

    /* Decode K and V once (they are shared by many rows). */
    const int64_t nkv = (int64_t)B * Hkv * S * D;
    double *K64 = (double *)malloc(sizeof(double) * (size_t)nkv);
    double *V64 = (double *)malloc(sizeof(double) * (size_t)nkv);
    if (!K64 || !V64) {
        free(K64);
        free(V64);
        return -2;
    }
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < nkv; ++t) {
        K64[t] = decode16(k[t], in_dtype);
        V64[t] = decode16(v[t], in_dtype);
    }

    const int g = Hq / Hkv;
    int err = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)S);
        double *q64 = (double *)malloc(sizeof(double) * (size_t)D);
        if (!s || !q64) {
#pragma omp atomic write
            err = -2;
        }
#pragma omp for schedule(dynamic, 4)
        for (int64_t t = 0; t < nrows; ++t) {
            if (!s || !q64)
                continue;
            const int64_t r = rows ? rows[t] : t;
            const int64_t i = r % S;
            const int64_t h = (r / S) % Hq;
            const int64_t b = r / ((int64_t)S * Hq);
            const int64_t hk = h / g;
            const int64_t nkeys = causal ? i + 1 : S;
            for (int d = 0; d < D; ++d)
                q64[d] = decode16(q[r * D + d], in_dtype);
            const double *Kh = K64 + (b * Hkv + hk) * (int64_t)S * D;
            const double *Vh = V64 + (b * Hkv + hk) * (int64_t)S * D;
            double lse_r;
            attn_row(q64, Kh, Vh, nkeys, D, scale, s, o + t * D, &lse_r);
            if (lse)
                lse[t] = lse_r;
        }
        free(s);
        free(q64);
    }
    free(K64);
    free(V64);
    return err;
}

/* ---- decode-time attention: Sq queries against Sk keys -------------------- */

/*
 * The paper's second workload (Section 6: "DC", a few new query positions against a long key/value
 * cache).  q,o [B][Hq][Sq][D]; k,v [B][Hkv][Sk][D]; lse [B][Hq][Sq] (may be NULL).  The Sq queries
 * are the LAST Sq positions of a sequence of Sk, so with `causal` query i sees keys
 * J_i = {0 .. Sk-Sq+i} (the diagonal is kept; Sk >= Sq is then required), and without it all Sk
 * keys.  Same three passes per row as above; Sq == Sk gives exactly the self-attention entry points.
 * Pinned (tests/test_oracle_pins.py) by: equality with the self-attention entry at Sq == Sk, equality
 * with the last Sq rows of a causal self-attention over Sk, the prefix property, a hand-expanded case,
 * V = 1 and Q = 0 closed forms.
 * Returns 0, -1 on bad arguments, -2 if memory cannot be had.
 */
int naut_oracle_attn_cross_f64(const double *q, const double *k, const double *v, double *o, double *lse,
                               int B, int Hq, int Hkv, int Sq, int Sk, int D, int causal, double scale)
{
    if (!q || !k || !v || !o || bad_shape(B, Hq, Hkv, Sq, D) || Sk <= 0 || (causal && Sk < Sq))
        return -1;
    const int g = Hq / Hkv;
    const int64_t nrows = (int64_t)B * Hq * Sq;
    int err = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)Sk);
        if (!s) {
#pragma omp atomic write
            err = -2;
        }
#pragma omp for schedule(dynamic, 4)
        for (int64_t r = 0; r < nrows; ++r) {
            if (!s)
                continue;
            const int64_t i = r % Sq;
            const int64_t h = (r / Sq) % Hq;
            const int64_t b = r / ((int64_t)Sq * Hq);
            const int64_t hk = h / g;
            const int64_t nkeys = causal ? (int64_t)Sk - Sq + i + 1 : Sk;
            const double *Kh = k + (b * Hkv + hk) * (int64_t)Sk * D;
            const double *Vh = v + (b * Hkv + hk) * (int64_t)Sk * D;
            double lse_r;
            attn_row(q + r * D, Kh, Vh, nkeys, D, scale, s, o + r * D, &lse_r);
            if (lse)
                lse[r] = lse_r;
        }
        free(s);
    }
    return err;
}

/* The same on bf16/fp16 bit patterns, decoded exactly. */
int naut_oracle_attn_cross16(const uint16_t *q, const uint16_t *k, const uint16_t *v, int in_dtype, double *o,
                             double *lse, int B, int Hq, int Hkv, int Sq, int Sk, int D, int causal,
                             double scale)
{
    if (!q || !k || !v || !o || bad_shape(B, Hq, Hkv, Sq, D) || Sk <= 0 || (causal && Sk < Sq))
        return -1;
    if (in_dtype != NAUT_ORACLE_BF16 && in_dtype != NAUT_ORACLE_F16)
        return -1;
    const int64_t nq = (int64_t)B * Hq * Sq * D, nkv = (int64_t)B * Hkv * Sk * D;
    double *Q64 = (double *)malloc(sizeof(double) * (size_t)nq);
    double *K64 = (double *)malloc(sizeof(double) * (size_t)nkv);
    double *V64 = (double *)malloc(sizeof(double) * (size_t)nkv);
    int rc = -2;
    if (Q64 && K64 && V64) {
        for (int64_t t = 0; t < nq; ++t)
            Q64[t] = decode16(q[t], in_dtype);
#pragma omp parallel for schedule(static)
        for (int64_t t = 0; t < nkv; ++t) {
            K64[t] = decode16(k[t], in_dtype);
            V64[t] = decode16(v[t], in_dtype);
        }
        rc = naut_oracle_attn_cross_f64(Q64, K64, V64, o, lse, B, Hq, Hkv, Sq, Sk, D, causal, scale);
    }
    free(Q64);
    free(K64);
    free(V64);
    return rc;
}

/* ---- FP8 (OCP E4M3) inputs ----------------------------------------------------- */

/*
 * OCP FP8 E4M3 ("e4m3fn"), the second input precision of the paper's experiments (Section 6): 1 sign,
 * 4 exponent bits (bias 7), 3 fraction bits; no infinities; exponent 15 with fraction 7 is NaN, every
 * other code is finite (largest 448); exponent 0 is subnormal with steps of 2^-9.
 */
static double decode_e4m3(uint8_t bits)
{
    const int sign = (bits >> 7) & 1;
    const int expo = (bits >> 3) & 0xf;
    const int frac = bits & 7;
    double mag;
    if (expo == 15 && frac == 7)
        mag = NAN;
    else if (expo == 0)
        mag = ldexp((double)frac, -9);
    else
        mag = ldexp(1.0 + (double)frac / 8.0, expo - 7);
    return sign ? -mag : mag;
}

int naut_oracle_decode_e4m3(const uint8_t *bits, double *out, int64_t n)
{
    if (!bits || !out || n < 0)
        return -1;
    for (int64_t t = 0; t < n; ++t)
        out[t] = decode_e4m3(bits[t]);
    return 0;
}

/*
 * Self-attention for a chosen list of query rows on FP8 inputs with per-tensor scales: the real
 * tensors are dq * decode(q), dk * decode(k), dv * decode(v) and the operator is the one above on
 * those real tensors.  Layouts and `rows` as in naut_oracle_attn_rows.  Pinned by the exhaustive
 * decode table against an independent library decode and by equality with the fp64 entry point on
 * the decoded, scaled inputs.
 */
int naut_oracle_attn_rows_e4m3(const uint8_t *q, const uint8_t *k, const uint8_t *v, double dq, double dk,
                               double dv, const int64_t *rows, int64_t nrows, double *o, double *lse, int B,
                               int Hq, int Hkv, int S, int D, int causal, double scale)
{
    if (!q || !k || !v || !o || bad_shape(B, Hq, Hkv, S, D) || nrows < 0)
        return -1;
    const int64_t total = (int64_t)B * Hq * S;
    if (!rows && nrows != total)
        return -1;
    if (rows)
        for (int64_t t = 0; t < nrows; ++t)
            if (rows[t] < 0 || rows[t] >= total)
                return -1;
    const int64_t nkv = (int64_t)B * Hkv * S * D;
    double *K64 = (double *)malloc(sizeof(double) * (size_t)nkv);
    double *V64 = (double *)malloc(sizeof(double) * (size_t)nkv);
    if (!K64 || !V64) {
        free(K64);
        free(V64);
        return -2;
    }
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < nkv; ++t) {
        K64[t] = dk * decode_e4m3(k[t]);
        V64[t] = dv * decode_e4m3(v[t]);
    }
    const int g = Hq / Hkv;
    int err = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)S);
        double *q64 = (double *)malloc(sizeof(double) * (size_t)D);
        if (!s || !q64) {
#pragma omp atomic write
            err = -2;
        }
#pragma omp for schedule(dynamic, 4)
        for (int64_t t = 0; t < nrows; ++t) {
            if (!s || !q64)
                continue;
            const int64_t r = rows ? rows[t] : t;
            const int64_t i = r % S;
            const int64_t h = (r / S) % Hq;
            const int64_t b = r / ((int64_t)S * Hq);
            const int64_t hk = h / g;
            const int64_t nkeys = causal ? i + 1 : S;
            for (int d = 0; d < D; ++d)
                q64[d] = dq * decode_e4m3(q[r * D + d]);
            const double *Kh = K64 + (b * Hkv + hk) * (int64_t)S * D;
            const double *Vh = V64 + (b * Hkv + hk) * (int64_t)S * D;
            double lse_r;
            attn_row(q64, Kh, Vh, nkeys, D, scale, s, o + t * D, &lse_r);
            if (lse)
                lse[t] = lse_r;
        }
        free(s);
        free(q64);
    }
    free(K64);
    free(V64);
    return err;
}

/* Exact decode of n 16-bit patterns to fp64 (exposed so tests can pin the decoders). */
int naut_oracle_decode16(const uint16_t *bits, int dtype, double *out, int64_t n)
{
    if (!bits || !out || n < 0 || (dtype != NAUT_ORACLE_BF16 && dtype != NAUT_ORACLE_F16))
        return -1;
    for (int64_t t = 0; t < n; ++t)
        out[t] = decode16(bits[t], dtype);
    return 0;
}

/* Number of threads the parallel regions above will use. */
int naut_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
