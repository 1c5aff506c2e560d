/*
 * naut_synth.c -- seeded synthetic Q/K/V generator (host only).
 *
 * Serves both the CPU oracle's tests and the GPU path's tests/benchmark with
 * identical bit patterns.  It contains none of the attention arithmetic: it only
 * draws iid N(0,1) samples and rounds them to bf16 / fp16 storage.
 *
 * The generator is counter based: the value of element `idx` of tensor `tag`
 * under `seed` depends on (seed, tag, idx) alone, so thread count and fill
 * order never matter.
 *
 *   key  = mix64(seed + GOLDEN * (tag + 1))
 *   h    = mix64(key + GOLDEN * (idx + 1))
 *   u1   = (hi32(h) + 0.5) / 2^32,  u2 = (lo32(h) + 0.5) / 2^32      (both in (0,1))
 *   z    = sqrt(-2 ln u1) * cos(2 pi u2)                              (Box-Muller)
 *   x    = (float)z * rowscale                                        (fp32)
 *   bits = round-to-nearest-even(x) in bf16 or fp16
 *
 * "Outlier rows" (the long-sequence workload scales 1 % of the K rows by 8 to
 * stress the running-max rescale): per (batch, head) the first `n_outlier`
 * entries of a seeded Fisher-Yates shuffle of 0..S-1 get rowscale = outlier_scale,
 * applied to the fp32 sample before rounding.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define NAUT_SYNTH_BF16 0
#define NAUT_SYNTH_F16 1

static const uint64_t GOLDEN = 0x9E3779B97F4A7C15ull;

/* splitmix64 finaliser */
static uint64_t mix64(uint64_t x)
{
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

static uint64_t stream_key(uint64_t seed, uint64_t tag)
{
    return mix64(seed + GOLDEN * (tag + 1));
}

static uint64_t draw(uint64_t key, uint64_t idx)
{
    return mix64(key + GOLDEN * (idx + 1));
}

static float normal_f32(uint64_t key, uint64_t idx)
{
    uint64_t h = draw(key, idx);
    double u1 = ((double)(h >> 32) + 0.5) * (1.0 / 4294967296.0);
    double u2 = ((double)(h & 0xffffffffull) + 0.5) * (1.0 / 4294967296.0);
    double z = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
    return (float)z;
}

/* fp32 -> bf16, round to nearest even (finite inputs; NaN is kept quiet). */
static uint16_t f32_to_bf16(float f)
{
    uint32_t w;
    memcpy(&w, &f, sizeof w);
    if ((w & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((w >> 16) | 0x0040u);
    uint32_t lsb = (w >> 16) & 1u;
    w += 0x7fffu + lsb;
    return (uint16_t)(w >> 16);
}

/* fp32 -> IEEE binary16, round to nearest even, with subnormals and overflow to inf. */
static uint16_t f32_to_f16(float f)
{
    uint32_t w;
    memcpy(&w, &f, sizeof w);
    uint32_t sign = (w >> 16) & 0x8000u;
    uint32_t a = w & 0x7fffffffu;
    if (a > 0x7f800000u)
        return (uint16_t)(sign | 0x7e00u); /* NaN */
    if (a >= 0x477ff000u)                  /* >= 65520 rounds to inf */
        return (uint16_t)(sign | 0x7c00u);
    if (a < 0x33000001u) /* <= 2^-25 rounds to zero (ties to even) */
        return (uint16_t)sign;
    int e = (int)(a >> 23) - 127;
    uint32_t man = (a & 0x7fffffu) | 0x800000u; /* 24-bit significand */
    int shift;                                  /* bits dropped from the significand */
    uint32_t base;
    if (e >= -14) {
        shift = 13;
        base = (uint32_t)(e + 15) << 10; /* exponent field; the implicit bit adds into it */
        man &= 0x7fffffu;
    } else {
        shift = 13 + (-14 - e); /* subnormal half */
        base = 0;
    }
    uint32_t kept = man >> shift;
    uint32_t rem = man & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (kept & 1u)))
        kept += 1; /* may carry into the exponent field: that is the right result */
    return (uint16_t)(sign | (base + kept));
}

static uint16_t round16(float f, int dtype)
{
    return dtype == NAUT_SYNTH_F16 ? f32_to_f16(f) : f32_to_bf16(f);
}

/*
 * First n entries of a seeded shuffle of 0..S-1 (distinct positions).
 * perm is caller scratch of S ints; the chosen positions are perm[0..n-1].
 */
static void pick_rows(uint64_t key, int S, int n, int32_t *perm)
{
    for (int i = 0; i < S; ++i)
        perm[i] = i;
    for (int t = 0; t < n; ++t) {
        uint64_t r = draw(key, (uint64_t)t);
        int j = t + (int)(r % (uint64_t)(S - t));
        int32_t tmp = perm[t];
        perm[t] = perm[j];
        perm[j] = tmp;
    }
}

/*
 * Fill out[B][H][S][D] with rounded N(0,1) samples.
 * n_outlier rows per (b,h) (0 <= n_outlier <= S) are multiplied by outlier_scale.
 * Returns 0, -1 on bad arguments, -2 on allocation failure.
 */
int naut_synth_fill(uint16_t *out, int B, int H, int S, int D, uint64_t seed, uint32_t tag, int dtype,
                    int n_outlier, float outlier_scale)
{
    if (!out || B <= 0 || H <= 0 || S <= 0 || D <= 0 || n_outlier < 0 || n_outlier > S)
        return -1;
    if (dtype != NAUT_SYNTH_BF16 && dtype != NAUT_SYNTH_F16)
        return -1;
    const uint64_t key = stream_key(seed, tag);
    const uint64_t okey = stream_key(seed, (uint64_t)tag + 0x10000u);
    int err = 0;
#pragma omp parallel
    {
        float *rowscale = (float *)malloc(sizeof(float) * (size_t)S);
        int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * (size_t)S);
        if (!rowscale || !perm) {
#pragma omp atomic write
            err = -2;
        }
#pragma omp for schedule(static)
        for (int64_t bh = 0; bh < (int64_t)B * H; ++bh) {
            if (!rowscale || !perm)
                continue;
            for (int i = 0; i < S; ++i)
                rowscale[i] = 1.0f;
            if (n_outlier > 0) {
                pick_rows(mix64(okey + GOLDEN * (uint64_t)(bh + 1)), S, n_outlier, perm);
                for (int t = 0; t < n_outlier; ++t)
                    rowscale[perm[t]] = outlier_scale;
            }
            for (int64_t i = 0; i < S; ++i)
                for (int64_t d = 0; d < D; ++d) {
                    int64_t idx = (bh * S + i) * D + d;
                    out[idx] = round16(normal_f32(key, (uint64_t)idx) * rowscale[i], dtype);
                }
        }
        free(rowscale);
        free(perm);
    }
    return err;
}

/* The outlier positions naut_synth_fill uses for (b,h) index bh; rows[n_outlier]. */
int naut_synth_outlier_rows(int32_t *rows, int64_t bh, int S, uint64_t seed, uint32_t tag, int n_outlier)
{
    if (!rows || S <= 0 || n_outlier < 0 || n_outlier > S || bh < 0)
        return -1;
    int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * (size_t)S);
    if (!perm)
        return -2;
    const uint64_t okey = stream_key(seed, (uint64_t)tag + 0x10000u);
    pick_rows(mix64(okey + GOLDEN * (uint64_t)(bh + 1)), S, n_outlier, perm);
    memcpy(rows, perm, sizeof(int32_t) * (size_t)n_outlier);
    free(perm);
    return 0;
}

/* Round n fp32 values to 16-bit storage (exposed for the rounding tests). */
int naut_synth_round16(const float *in, uint16_t *out, int64_t n, int dtype)
{
    if (!in || !out || n < 0 || (dtype != NAUT_SYNTH_BF16 && dtype != NAUT_SYNTH_F16))
        return -1;
    for (int64_t t = 0; t < n; ++t)
        out[t] = round16(in[t], dtype);
    return 0;
}

/*
 * Round n floats to OCP FP8 E4M3 ("e4m3fn": 1 sign, 4 exponent bits with bias 7, 3 fraction bits, no
 * infinities, largest finite value 448), to nearest with ties to even, magnitudes beyond 448 saturating
 * to 448.  Inputs must be finite.  Used to store the synthetic Q, K, V of the FP8 workloads.
 */
int naut_synth_round_e4m3(const float *in, uint8_t *out, int64_t n)
{
    if (!in || !out || n < 0)
        return -1;
    for (int64_t t = 0; t < n; ++t) {
        const float x = in[t];
        const uint8_t sign = signbit(x) ? 0x80 : 0x00;
        const float a = fabsf(x);
        uint8_t code;
        if (!(a < 464.0f)) {          /* 464 is the midpoint between 448 and the first value not representable */
            code = 0x7e;
        } else if (a < 0.015625f) {   /* below 2^-6: subnormal steps of 2^-9 (8 steps reach the first normal code) */
            code = (uint8_t)rintf(a * 512.0f);
        } else {
            int e;
            (void)frexpf(a, &e);      /* a = f * 2^e, f in [0.5, 1)  ->  a = (1 + m/8) * 2^(e-1) */
            int E = e - 1;
            int m = (int)rintf(ldexpf(a, -E) * 8.0f) - 8;
            if (m == 8) {
                m = 0;
                E += 1;
            }
            const int c = ((E + 7) << 3) | m;
            code = (uint8_t)(c > 0x7e ? 0x7e : c);
        }
        out[t] = sign | code;
    }
    return 0;
}
