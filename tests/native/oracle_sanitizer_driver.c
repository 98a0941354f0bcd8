/*
 * The CPU oracle under the address and undefined-behaviour sanitizers: every entry point on
 * small inputs held in exact-size heap buffers (an access one element beyond any of them is
 * reported), with results that are known in closed form because every value is a small
 * integer or a power of two (all sums are exact).  Built and run by tests/test_host_tables.py
 * together with oracle/adafuse_oracle.c.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double oracle_bf16_to_f64(uint16_t bits);
uint16_t oracle_f64_to_bf16_rne(double x);
int oracle_pregate(const uint16_t *, const uint16_t *, int, int, int, int, int, double *, float *, int32_t *, double *, float *);
int oracle_merge_rows(const uint16_t *, int64_t, const uint16_t *, const uint16_t *, int, int, int, int, const int32_t *,
                      const float *, int, float, int, int, uint16_t *, int64_t);
int oracle_merge_rows_f64(const uint16_t *, int64_t, const uint16_t *, const uint16_t *, int, int, int, int, const int32_t *,
                          const float *, int, float, int, int, double *, int64_t);
int oracle_inplace_swap_rows(const uint16_t *, int64_t, const uint16_t *, const uint16_t *, int, int, int, int, const int32_t *,
                             const float *, int, const int32_t *, const float *, int, float, int, int, uint16_t *, int64_t);
int oracle_dynamic_adapter_forward(const uint16_t *, int64_t, const uint16_t *, const uint16_t *, int, int, int, int,
                                   const int32_t *, const float *, int, float, const double *, double *);
int oracle_gemv_bf16(const uint16_t *, int64_t, int, int, const double *, double *);
int oracle_bf16_ulp_diff(const uint16_t *, const uint16_t *, int64_t, int64_t *, int64_t *);

static int fails = 0;
#define CHECK(c) do { if (!(c)) { printf("FAIL line %d: %s\n", __LINE__, #c); ++fails; } } while (0)

static uint16_t bf(double x) { return oracle_f64_to_bf16_rne(x); }

int main(void)
{
    enum { OUT = 5, IN = 7, LDW = 9, E = 3, R = 2 };
    /* rounding: exact values, a tie to even, the value just above the tie */
    CHECK(bf(1.0) == 0x3F80 && bf(-2.0) == 0xC000 && bf(0.0) == 0x0000);
    CHECK(bf(1.0 + ldexp(1.0, -8)) == 0x3F80);                     /* halfway between 1 and 1 + 2^-7: to even */
    CHECK(bf(1.0 + ldexp(1.0, -8) + ldexp(1.0, -40)) == 0x3F81);
    CHECK(bf(1.0 + 3 * ldexp(1.0, -8)) == 0x3F82);                 /* halfway between odd and even: to even (up) */
    CHECK(oracle_bf16_to_f64(0x3F81) == 1.0 + ldexp(1.0, -7));

    uint16_t *w = malloc(sizeof(uint16_t) * OUT * LDW), *a = malloc(sizeof(uint16_t) * E * R * IN),
             *b = malloc(sizeof(uint16_t) * E * OUT * R), *res = malloc(sizeof(uint16_t) * OUT * IN);
    double *resf = malloc(sizeof(double) * OUT * IN), *x = malloc(sizeof(double) * IN), *y = malloc(sizeof(double) * OUT),
           *y2 = malloc(sizeof(double) * OUT);
    for (int o = 0; o < OUT; ++o)
        for (int i = 0; i < LDW; ++i) w[o * LDW + i] = i < IN ? bf(o - i) : 0x7FC1;   /* padding columns: NaN, never read */
    for (int e = 0; e < E; ++e)
        for (int p = 0; p < R; ++p)
            for (int i = 0; i < IN; ++i) a[(e * R + p) * IN + i] = bf((e + 1) * (p + 1) + i);
    for (int e = 0; e < E; ++e)
        for (int o = 0; o < OUT; ++o)
            for (int p = 0; p < R; ++p) b[(e * OUT + o) * R + p] = bf(o - p - e);
    for (int i = 0; i < IN; ++i) x[i] = i - 3;

    /* merge: W + s * sum_j g_j B_j A_j with s = 2, experts 2 and 0, gates 0.5 and 0.25 */
    const int32_t idx[2] = {2, 0};
    const float gates[2] = {0.5f, 0.25f};
    CHECK(oracle_merge_rows_f64(w, LDW, a, b, OUT, IN, E, R, idx, gates, 2, 2.0f, 0, OUT, resf, IN) == 0);
    CHECK(oracle_merge_rows(w, LDW, a, b, OUT, IN, E, R, idx, gates, 2, 2.0f, 0, OUT, res, IN) == 0);
    for (int o = 0; o < OUT; ++o)
        for (int i = 0; i < IN; ++i) {
            double want = o - i;
            for (int j = 0; j < 2; ++j)
                for (int p = 0; p < R; ++p) want += 2.0 * gates[j] * (o - p - idx[j]) * ((idx[j] + 1) * (p + 1) + i);
            CHECK(resf[o * IN + i] == want);
            CHECK(res[o * IN + i] == bf(want));
        }
    /* rows [1, 3) only, into a buffer of exactly that size */
    uint16_t *part = malloc(sizeof(uint16_t) * 2 * IN);
    CHECK(oracle_merge_rows(w, LDW, a, b, OUT, IN, E, R, idx, gates, 2, 2.0f, 1, 3, part, IN) == 0);
    CHECK(memcmp(part, res + IN, sizeof(uint16_t) * 2 * IN) == 0);
    /* no expert, and zero gates: the base weights come back bit for bit */
    const float zeros[2] = {0.0f, 0.0f};
    CHECK(oracle_merge_rows(w, LDW, a, b, OUT, IN, E, R, idx, zeros, 2, 2.0f, 0, OUT, res, IN) == 0);
    for (int o = 0; o < OUT; ++o) CHECK(memcmp(res + o * IN, w + o * LDW, sizeof(uint16_t) * IN) == 0);
    CHECK(oracle_merge_rows(w, LDW, NULL, NULL, OUT, IN, E, R, NULL, NULL, 0, 2.0f, 0, OUT, res, IN) == 0);
    for (int o = 0; o < OUT; ++o) CHECK(memcmp(res + o * IN, w + o * LDW, sizeof(uint16_t) * IN) == 0);
    /* an expert index outside the bank is refused, not read */
    const int32_t bad[2] = {3, 0};
    CHECK(oracle_merge_rows(w, LDW, a, b, OUT, IN, E, R, bad, gates, 2, 2.0f, 0, OUT, res, IN) != 0);

    /* in-place step: removing and re-adding the same experts is the identity (all values exact) */
    uint16_t *cur = malloc(sizeof(uint16_t) * OUT * IN);
    CHECK(oracle_merge_rows(w, LDW, a, b, OUT, IN, E, R, idx, gates, 2, 2.0f, 0, OUT, cur, IN) == 0);
    CHECK(oracle_inplace_swap_rows(cur, IN, a, b, OUT, IN, E, R, idx, gates, 2, idx, gates, 2, 2.0f, 0, OUT, res, IN) == 0);
    CHECK(memcmp(res, cur, sizeof(uint16_t) * OUT * IN) == 0);
    /* ... and removing them alone gives the base weights back */
    CHECK(oracle_inplace_swap_rows(cur, IN, a, b, OUT, IN, E, R, idx, gates, 2, NULL, NULL, 0, 2.0f, 0, OUT, res, IN) == 0);
    for (int o = 0; o < OUT; ++o) CHECK(memcmp(res + o * IN, w + o * LDW, sizeof(uint16_t) * IN) == 0);

    /* forward: the dynamic-adapter output equals the mat-vec with the (exactly representable) merged weights */
    CHECK(oracle_dynamic_adapter_forward(w, LDW, a, b, OUT, IN, E, R, idx, gates, 2, 2.0f, x, y) == 0);
    for (int o = 0; o < OUT; ++o) {
        double s = 0;
        for (int i = 0; i < IN; ++i) s += resf[o * IN + i] * x[i];
        CHECK(y[o] == s);
    }
    CHECK(oracle_gemv_bf16(w, LDW, OUT, IN, x, y2) == 0);
    for (int o = 0; o < OUT; ++o) {
        double s = 0;
        for (int i = 0; i < IN; ++i) s += (o - i) * x[i];
        CHECK(y2[o] == s);
    }

    /* router: 2 tokens, 4 experts, d = 3; token 1 has an exact tie between experts 1 and 3 */
    enum { T = 2, D = 3, NE = 4, K = 2 };
    uint16_t *h = malloc(sizeof(uint16_t) * T * D), *wr = malloc(sizeof(uint16_t) * NE * D);
    const double hv[T][D] = {{1, 0, 2}, {0, 1, 0}}, wv[NE][D] = {{1, 0, 0}, {0, 2, 1}, {3, 0, -1}, {5, 2, -2}};
    for (int t = 0; t < T; ++t) for (int i = 0; i < D; ++i) h[t * D + i] = bf(hv[t][i]);
    for (int e = 0; e < NE; ++e) for (int i = 0; i < D; ++i) wr[e * D + i] = bf(wv[e][i]);
    double *lg = malloc(sizeof(double) * T * NE), *g = malloc(sizeof(double) * T * K);
    float *lg32 = malloc(sizeof(float) * T * NE), *g32 = malloc(sizeof(float) * T * K);
    int32_t *sel = malloc(sizeof(int32_t) * T * K);
    CHECK(oracle_pregate(h, wr, T, D, NE, K, 0, lg, lg32, sel, g, g32) == 0);
    /* token 0 logits: 1, 2, 1, 1 -> experts 1 then 0 (tie among 0, 2, 3: lowest index); token 1: 0, 2, 0, 2 -> 1 then 3 */
    CHECK(lg[0] == 1 && lg[1] == 2 && lg[2] == 1 && lg[3] == 1 && lg[4] == 0 && lg[5] == 2 && lg[6] == 0 && lg[7] == 2);
    CHECK(sel[0] == 1 && sel[1] == 0 && sel[2] == 1 && sel[3] == 3);
    CHECK(fabs(g[0] - 1.0 / (1.0 + exp(-1.0))) < 1e-15 && fabs(g[0] + g[1] - 1.0) < 1e-15);
    CHECK(g[2] == 0.5 && g[3] == 0.5 && g32[2] == 0.5f);
    CHECK(oracle_pregate(h, wr, T, D, NE, K, 1, NULL, NULL, sel, g, NULL) == 0);   /* softmax over all four, keep two */
    CHECK(fabs(g[2] - 1.0 / (2.0 + 2.0 * exp(-2.0))) < 1e-15);

    int64_t mx = 0, nd = 0;
    const uint16_t p[4] = {0x3F80, 0x3F81, 0x8000, 0x0001}, q[4] = {0x3F80, 0x3F83, 0x0000, 0x8001};
    CHECK(oracle_bf16_ulp_diff(p, q, 4, &mx, &nd) == 0 && mx == 2 && nd == 2);       /* -0 and +0 coincide */

    free(w); free(a); free(b); free(res); free(resf); free(x); free(y); free(y2); free(part); free(cur);
    free(h); free(wr); free(lg); free(g); free(lg32); free(g32); free(sel);
    if (fails) { printf("%d checks failed\n", fails); return 1; }
    printf("oracle under sanitizers ok\n");
    return 0;
}
