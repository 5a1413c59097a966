/*
 * CPU oracle for the MixLLM quantized linear layer (arxiv 2412.14590).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
 * GPU library computes.  Only the test-suite, the smoke check and the
 * `cpu_baseline` leg of the benchmark may call it; the product path never does.
 * It shares no code, header, table or helper with the HIP sources.
 *
 * Everything works on canonical, unpacked layouts:
 *   W        fp16 bit patterns, [rows, K] row-major
 *   q4       one uint4 code per byte, [rows, K]
 *   z4       one uint4 zero point per byte, [rows, K/G]
 *   s4 / s8  fp16 bit patterns, [rows, K/G] (s8: [rows, K/w8_group])
 *   q8, xq   int8, row-major
 *   xs       fp16 bit patterns, [M, K/act_group]
 *   perm     int32 [N]: row j of the concatenation [8-bit rows ; 4-bit rows]
 *            is output channel perm[j]
 *
 * What each function follows:
 *   - quantizers: the uniform affine quantizer X_q = clamp(round(X/s)+z, range)
 *     of Sec. 2, with the configuration of Sec. 3.1.2 / Sec. 4.1 (8-bit
 *     symmetric, 4-bit asymmetric, groups of G along K).  Points the paper is
 *     silent on (how s and z are derived, tie-break, int8 range, degenerate
 *     groups) take these readings: min/max with the range widened to contain
 *     0, round-half-to-even, int8 range [-127,127], scale 1 when the computed
 *     scale is 0, scales stored as fp16 and used as such by the quantizer.
 *   - group partials and the linear: the two-step dequantization of Sec. 3.3,
 *     Y = ((W_q - z) x A_q) . s_w . s_a per group (Sec. 3.5), summed over groups.
 *   - scatter: both parts write one output tensor at their own channel indices
 *     (Sec. 3.4).
 *   - channel salience and the global choice of the 8-bit channels: Sec. 3.2, Eq. 4 and
 *     Alg. 1 (equal saliences: the earlier channel first).
 *
 * Quantizer arithmetic is IEEE binary32 (true division, rintf under the default
 * round-to-nearest-even mode), inputs widened exactly from fp16; the linear
 * accumulates in binary64 and rounds once to fp16.
 *
 * Parity pins (CPU tests): brute-force fp64 dequantize-then-matmul on small
 * inputs, closed forms, invariants, the analytic rounding-error bound, and an
 * exhaustive check of the fp16 conversions against numpy.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ fp16 -- */

/* fp16 bit pattern -> double (exact). */
static double h2d(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);               /* zero / subnormal */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m + 1024), e - 25);   /* (1 + m/1024) * 2^(e-15) */
    return sign ? -v : v;
}

static float h2f(uint16_t h) { return (float)h2d(h); }   /* exact: fp16 subset of fp32 */

/* double -> fp16 bit pattern, one rounding, ties to even, overflow to inf. */
static uint16_t d2h(double v)
{
    uint16_t sign = signbit(v) ? 0x8000u : 0u;
    double a = fabs(v);
    if (isnan(v)) return 0x7e00u;
    if (a == 0.0) return sign;
    if (isinf(a)) return (uint16_t)(sign | 0x7c00u);
    int e;
    (void)frexp(a, &e);               /* a = f * 2^e, f in [0.5,1): leading bit 2^(e-1) */
    int E = e - 1;
    if (E < -14) E = -14;             /* subnormal range shares the spacing 2^-24 */
    double ulp = ldexp(1.0, E - 10);
    double n = nearbyint(a / ulp);    /* power-of-two quotient is exact; ties-to-even */
    double r = n * ulp;               /* rounded magnitude */
    if (r >= 65536.0) return (uint16_t)(sign | 0x7c00u);
    if (r < ldexp(1.0, -14)) return (uint16_t)(sign | (uint16_t)ldexp(r, 24));
    (void)frexp(r, &e);
    E = e - 1;
    int mant = (int)ldexp(r, 10 - E) - 1024;
    return (uint16_t)(sign | (uint16_t)((E + 15) << 10) | (uint16_t)mant);
}

/* exported so the tests can pin the conversions against numpy */
void oracle_half_to_double(const uint16_t *h, int64_t n, double *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = h2d(h[i]);
}
void oracle_double_to_half(const double *v, int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = d2h(v[i]);
}

static float clampf(float v, float lo, float hi) { return v < lo ? lo : (v > hi ? hi : v); }

/* fp32 scale -> the stored fp16 scale; a scale that is (or rounds to) zero becomes 1. */
static uint16_t store_scale(float s32)
{
    uint16_t s16 = d2h((double)s32);
    if ((s16 & 0x7fffu) == 0) s16 = 0x3c00u;   /* 1.0 */
    return s16;
}

/* ------------------------------------------------------------ quantizers -- */

/* Symmetric int8 quantization of `rows` vectors, one scale per `group` consecutive
 * elements (group == K gives per-token / per-channel).  Sec. 2 formula with z = 0. */
static void quantize_sym8(const uint16_t *X, int64_t rows, int64_t K, int64_t group,
                          int8_t *q, uint16_t *s)
{
    int64_t ng = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t g = 0; g < ng; ++g) {
            const uint16_t *x = X + r * K + g * group;
            float amax = 0.0f;
            for (int64_t k = 0; k < group; ++k) {
                float a = fabsf(h2f(x[k]));
                if (a > amax) amax = a;
            }
            uint16_t s16 = store_scale(amax / 127.0f);
            float sc = h2f(s16);
            s[r * ng + g] = s16;
            for (int64_t k = 0; k < group; ++k) {
                float t = rintf(h2f(x[k]) / sc);
                q[r * K + g * group + k] = (int8_t)clampf(t, -127.0f, 127.0f);
            }
        }
    }
}

/* Activations: int8 symmetric; act_group == K is per token, act_group == G is the
 * group-wise configuration of Sec. 3.1.2. */
void oracle_quantize_act(const uint16_t *x, int64_t M, int64_t K, int64_t act_group,
                         int8_t *xq, uint16_t *xs)
{
    quantize_sym8(x, M, K, act_group, xq, xs);
}

/* 8-bit weight rows: int8 symmetric; w8_group == K is per channel, == G group-wise. */
void oracle_quantize_w8(const uint16_t *W, int64_t rows, int64_t K, int64_t w8_group,
                        int8_t *q, uint16_t *s)
{
    quantize_sym8(W, rows, K, w8_group, q, s);
}

/* 4-bit weight rows: asymmetric uint4 per (row, group of G). */
void oracle_quantize_w4(const uint16_t *W, int64_t rows, int64_t K, int64_t G,
                        uint8_t *q, uint16_t *s, uint8_t *z)
{
    int64_t ng = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t g = 0; g < ng; ++g) {
            const uint16_t *w = W + r * K + g * G;
            float mn = 0.0f, mx = 0.0f;          /* range always contains 0 */
            for (int64_t k = 0; k < G; ++k) {
                float v = h2f(w[k]);
                if (v < mn) mn = v;
                if (v > mx) mx = v;
            }
            uint16_t s16 = store_scale((mx - mn) / 15.0f);
            float sc = h2f(s16);
            float zf = clampf(rintf(-mn / sc), 0.0f, 15.0f);
            s[r * ng + g] = s16;
            z[r * ng + g] = (uint8_t)zf;
            for (int64_t k = 0; k < G; ++k) {
                float t = rintf(h2f(w[k]) / sc) + zf;
                q[r * K + g * G + k] = (uint8_t)clampf(t, 0.0f, 15.0f);
            }
        }
    }
}

/* Order of the concatenated rows: the n8 salient channels in ascending order,
 * then every other channel in ascending order (Sec. 3.4 only says the two parts
 * own different channel indices; this order is the reading used throughout).
 * Returns 0, or -1 if salient_idx has a duplicate or an index outside [0,N). */
int oracle_feature_perm(int64_t N, int64_t n8, const int32_t *salient_idx, int32_t *perm)
{
    uint8_t *mark = (uint8_t *)calloc((size_t)(N > 0 ? N : 1), 1);
    if (!mark) return -2;
    for (int64_t i = 0; i < n8; ++i) {
        int32_t c = salient_idx[i];
        if (c < 0 || c >= N || mark[c]) { free(mark); return -1; }
        mark[c] = 1;
    }
    int64_t a = 0, b = n8;
    for (int64_t c = 0; c < N; ++c) {
        if (mark[c]) perm[a++] = (int32_t)c;
        else         perm[b++] = (int32_t)c;
    }
    free(mark);
    return 0;
}

/* ------------------------------------------------- partials and the linear -- */

/* Exact integer dot product of one activation row with one weight row over one
 * group: sum_k a[k] * (w[k] - z).  For an 8-bit row z = 0 and w is int8. */
static int32_t dot_group4(const int8_t *a, const uint8_t *w, int z, int64_t G)
{
    int32_t acc = 0;
    for (int64_t k = 0; k < G; ++k) acc += (int32_t)a[k] * ((int32_t)w[k] - z);
    return acc;
}
static int32_t dot_group8(const int8_t *a, const int8_t *w, int64_t G)
{
    int32_t acc = 0;
    for (int64_t k = 0; k < G; ++k) acc += (int32_t)a[k] * (int32_t)w[k];
    return acc;
}

/* P[m, perm[j], g] = sum_{k in group g} xq[m,k] * (row j's integer weight)  (Sec. 3.3,
 * step 1 of the two-step dequantization followed by the int8 MatMul of one group).
 * P is [M, N, K/G] in ORIGINAL channel order. */
void oracle_group_partials(const int8_t *xq, const int8_t *q8, const uint8_t *q4,
                           const uint8_t *z4, const int32_t *perm,
                           int64_t M, int64_t K, int64_t N, int64_t n8, int64_t G,
                           int32_t *P)
{
    int64_t ng = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < N; ++j) {
        int64_t c = perm[j];
        for (int64_t m = 0; m < M; ++m) {
            for (int64_t g = 0; g < ng; ++g) {
                const int8_t *a = xq + m * K + g * G;
                int32_t p;
                if (j < n8) {
                    p = dot_group8(a, q8 + j * K + g * G, G);
                } else {
                    int64_t r = j - n8;
                    p = dot_group4(a, q4 + r * K + g * G, z4[r * ng + g], G);
                }
                P[(m * N + c) * ng + g] = p;
            }
        }
    }
}

/* y[m, perm[j]] = fp16( sum_g P[m,j,g] * s_w[j,g] * s_a[m,g] ), the sum and the
 * products in binary64 (Sec. 3.3 step 2; closed form in Sec. 3.5; scatter Sec. 3.4).
 * s8 is [n8, K/w8_group], xs is [M, K/act_group]; a group g uses the scale of the
 * (coarser) block that contains it.  y64 (optional, may be NULL) receives the
 * unrounded sums, [M,N]. */
void oracle_mixed_linear(const int8_t *xq, const uint16_t *xs, int64_t act_group,
                         const int8_t *q8, const uint16_t *s8, int64_t w8_group,
                         const uint8_t *q4, const uint16_t *s4, const uint8_t *z4,
                         const int32_t *perm,
                         int64_t M, int64_t K, int64_t N, int64_t n8, int64_t G,
                         uint16_t *y, double *y64)
{
    int64_t ng = K / G;
    int64_t nga = K / act_group, ng8 = K / w8_group;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < N; ++j) {
        int64_t c = perm[j];
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int64_t g = 0; g < ng; ++g) {
                const int8_t *a = xq + m * K + g * G;
                double sa = h2d(xs[m * nga + (g * G) / act_group]);
                double sw;
                int32_t p;
                if (j < n8) {
                    p = dot_group8(a, q8 + j * K + g * G, G);
                    sw = h2d(s8[j * ng8 + (g * G) / w8_group]);
                } else {
                    int64_t r = j - n8;
                    p = dot_group4(a, q4 + r * K + g * G, z4[r * ng + g], G);
                    sw = h2d(s4[r * ng + g]);
                }
                acc += (double)p * sw * sa;
            }
            if (y64) y64[m * N + c] = acc;
            y[m * N + c] = d2h(acc);
        }
    }
}

/* ---- global precision search (Sec. 3.2) ------------------------------------------------- */

/* Salience of every output channel of one layer for one gradient sample (Eq. 4 with a single
 * sample d; lines 3-6 of Alg. 1):
 *     S1[n] = sum_k G[n][k] * (Qdq(W)[n][k] - W[n][k]),    S[n] = | S1[n] + S1[n]^2 / 2 |
 * where Qdq is the 4-bit group-wise quantizer above followed by its dequantization
 * (q - z) * s.  The sum runs in double.  salience[n] = (accumulate ? salience[n] : 0) + weight * S[n]:
 * Eq. 4's mean over the calibration set is one call per sample with weight = 1 / |D|.
 * s1 (may be NULL) receives S1 of this sample. */
void oracle_channel_salience(const uint16_t *W, const uint16_t *Gr, int64_t N, int64_t K, int64_t G,
                             double weight, int accumulate, double *salience, double *s1)
{
    int64_t ng = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        uint8_t *q = (uint8_t *)malloc((size_t)K);
        uint16_t *s = (uint16_t *)malloc((size_t)ng * sizeof(uint16_t));
        uint8_t *z = (uint8_t *)malloc((size_t)ng);
        oracle_quantize_w4(W + n * K, 1, K, G, q, s, z);
        double first = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            int64_t g = k / G;
            double deq = ((double)q[k] - (double)z[g]) * h2d(s[g]);
            first += h2d(Gr[n * K + k]) * (deq - h2d(W[n * K + k]));
        }
        double sal = fabs(first + 0.5 * first * first);
        if (s1) s1[n] = first;
        salience[n] = (accumulate ? salience[n] : 0.0) + weight * sal;
        free(q); free(s); free(z);
    }
}

/* Last two lines of Alg. 1: all channels of all layers (saliences concatenated, `total` of
 * them) sorted by salience, descending; the first T are marked.  The paper does not say how
 * equal saliences are ordered: the channel that comes first in the concatenation wins. */
typedef struct { float s; int64_t i; } sal_item;
static int sal_cmp(const void *a, const void *b)
{
    const sal_item *x = (const sal_item *)a, *y = (const sal_item *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return x->i < y->i ? -1 : (x->i > y->i ? 1 : 0);
}
int oracle_select_salient(const float *salience, int64_t total, int64_t T, uint8_t *chosen)
{
    if (T < 0 || T > total) return -1;
    sal_item *it = (sal_item *)malloc((size_t)(total > 0 ? total : 1) * sizeof(sal_item));
    if (!it) return -2;
    for (int64_t i = 0; i < total; ++i) { it[i].s = salience[i]; it[i].i = i; chosen[i] = 0; }
    qsort(it, (size_t)total, sizeof(sal_item), sal_cmp);
    for (int64_t i = 0; i < T; ++i) chosen[it[i].i] = 1;
    free(it);
    return 0;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
