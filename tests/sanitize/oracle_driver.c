/* Runs every function of the CPU oracle on exactly-sized heap buffers, ragged shapes included,
 * in a build with -fsanitize=address,undefined: an access outside a buffer, a signed overflow, a
 * misaligned or invalid conversion aborts the run.  Test infrastructure (built and run by
 * tests/test_sanitizers.py); the values are also checked against a few invariants so that the
 * calls cannot be optimised away. */
#include "../../oracle/mixllm_oracle.c"

#include <stdio.h>
#include <string.h>

static uint32_t rng_state = 12345u;
static uint32_t rnd(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state >> 8;
}
/* a finite fp16 bit pattern of moderate magnitude, both signs, some zeros and subnormals */
static uint16_t rnd_half(void)
{
    uint32_t r = rnd();
    if ((r & 63) == 0) return 0;
    if ((r & 63) == 1) return (uint16_t)(r >> 8 & 0x3ff);         /* subnormal */
    return (uint16_t)(((r >> 6) & 0x8000) | ((8 + (r >> 10) % 12) << 10) | ((r >> 14) & 0x3ff));
}
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "oracle_driver: check failed at line %d: %s\n", __LINE__, #c); return 1; } } while (0)

static int run_case(int64_t M, int64_t K, int64_t N, int64_t n8, int64_t act_group, int64_t w8_group)
{
    const int64_t G = 128, ng = K / G, n4 = N - n8;
    uint16_t *W = malloc((size_t)(N * K) * 2), *x = malloc((size_t)(M * K + 1) * 2);
    for (int64_t i = 0; i < N * K; ++i) W[i] = rnd_half();
    for (int64_t i = 0; i < M * K; ++i) x[i] = rnd_half();
    int32_t *sal = malloc((size_t)(n8 + 1) * 4), *perm = malloc((size_t)N * 4);
    for (int64_t i = 0; i < n8; ++i) sal[i] = (int32_t)((i * 7 + 3) % N);   /* distinct while n8 <= N and gcd(7, N) = 1 */
    int rc = oracle_feature_perm(N, n8, sal, perm);
    if (rc != 0) {   /* 7 divides N: take the first n8 channels instead */
        for (int64_t i = 0; i < n8; ++i) sal[i] = (int32_t)i;
        CHECK(oracle_feature_perm(N, n8, sal, perm) == 0);
    }
    /* gather rows into the two parts */
    uint16_t *W8 = malloc((size_t)(n8 * K + 1) * 2), *W4 = malloc((size_t)(n4 * K + 1) * 2);
    for (int64_t j = 0; j < N; ++j)
        memcpy(j < n8 ? W8 + j * K : W4 + (j - n8) * K, W + (int64_t)perm[j] * K, (size_t)K * 2);
    int8_t *q8 = malloc((size_t)(n8 * K + 1)), *xq = malloc((size_t)(M * K + 1));
    uint16_t *s8 = malloc((size_t)(n8 * (K / w8_group) + 1) * 2), *xs = malloc((size_t)(M * (K / act_group) + 1) * 2);
    uint8_t *q4 = malloc((size_t)(n4 * K + 1)), *z4 = malloc((size_t)(n4 * ng + 1));
    uint16_t *s4 = malloc((size_t)(n4 * ng + 1) * 2);
    oracle_quantize_w8(W8, n8, K, w8_group, q8, s8);
    oracle_quantize_w4(W4, n4, K, G, q4, s4, z4);
    oracle_quantize_act(x, M, K, act_group, xq, xs);
    for (int64_t i = 0; i < n4 * K; ++i) CHECK(q4[i] <= 15);
    for (int64_t i = 0; i < n4 * ng; ++i) CHECK(z4[i] <= 15);
    for (int64_t i = 0; i < M * K; ++i) CHECK(xq[i] >= -127);
    int32_t *P = malloc((size_t)(M * N * ng + 1) * 4);
    oracle_group_partials(xq, q8, q4, z4, perm, M, K, N, n8, G, P);
    uint16_t *y = malloc((size_t)(M * N + 1) * 2);
    double *y64 = malloc((size_t)(M * N + 1) * 8);
    oracle_mixed_linear(xq, xs, act_group, q8, s8, w8_group, q4, s4, z4, perm, M, K, N, n8, G, y, y64);
    oracle_mixed_linear(xq, xs, act_group, q8, s8, w8_group, q4, s4, z4, perm, M, K, N, n8, G, y, NULL);
    double *back = malloc((size_t)(M * N + 1) * 8);
    oracle_half_to_double(y, M * N, back);
    uint16_t *again = malloc((size_t)(M * N + 1) * 2);
    oracle_double_to_half(y64, M * N, again);
    for (int64_t i = 0; i < M * N; ++i) CHECK(again[i] == y[i]);
    /* global precision search on the same weights, x standing in for a gradient where shapes allow */
    double *salience = malloc((size_t)N * 8), *s1 = malloc((size_t)N * 8);
    oracle_channel_salience(W, W, N, K, G, 0.5, 0, salience, s1);
    oracle_channel_salience(W, W, N, K, G, 0.5, 1, salience, NULL);
    float *sf = malloc((size_t)N * 4);
    uint8_t *chosen = malloc((size_t)N);
    for (int64_t i = 0; i < N; ++i) sf[i] = (float)salience[i];
    CHECK(oracle_select_salient(sf, N, n8, chosen) == 0);
    int64_t cnt = 0;
    for (int64_t i = 0; i < N; ++i) cnt += chosen[i];
    CHECK(cnt == n8);
    CHECK(oracle_select_salient(sf, N, N + 1, chosen) == -1);
    free(W); free(x); free(sal); free(perm); free(W8); free(W4); free(q8); free(xq); free(s8); free(xs); free(q4);
    free(z4); free(s4); free(P); free(y); free(y64); free(back); free(again); free(salience); free(s1); free(sf); free(chosen);
    return 0;
}

int main(void)
{
    static const int64_t shapes[][4] = {{1, 128, 1, 0}, {1, 128, 1, 1}, {3, 256, 7, 2}, {5, 384, 33, 33}, {2, 640, 50, 0},
                                        {17, 1024, 100, 9}, {4, 2048, 31, 5}};
    for (size_t i = 0; i < sizeof(shapes) / sizeof(shapes[0]); ++i) {
        const int64_t M = shapes[i][0], K = shapes[i][1], N = shapes[i][2], n8 = shapes[i][3];
        if (run_case(M, K, N, n8, K, K)) return 1;
        if (run_case(M, K, N, n8, 128, 128)) return 1;
        if (run_case(M, K, N, n8, K, 128)) return 1;
    }
    /* bad lists are refused, not read past */
    int32_t dup[2] = {1, 1}, far[1] = {9}, perm[4];
    if (oracle_feature_perm(4, 2, dup, perm) != -1 || oracle_feature_perm(4, 1, far, perm) != -1) return 1;
    printf("oracle_driver: ok (%d threads)\n", oracle_num_threads());
    return 0;
}
