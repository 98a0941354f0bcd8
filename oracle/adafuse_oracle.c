/*
 * AdaFuse CPU oracle -- TEST INFRASTRUCTURE, not a product path.
 *
 * A plain, slow, fp64 statement of what the pre-gating router and the fused
 * adapter switch compute, written from the paper's definitions.  Nothing here
 * is shared with the HIP kernels (no header, table, helper or constant), and
 * only tests, the smoke check and the bench's cpu_baseline leg may call it.
 *
 * Conventions (paper gives no shapes; these follow E(x) = W_up(W_down x) of
 * Eq.1 in the y = W x convention):
 *   W      [out][ldw]   bf16 bit patterns (uint16), row-major, ldw >= in
 *   A bank [E][r][in]   bf16, expert e's LoRA_DOWN  (A_e = W_down)
 *   B bank [E][out][r]  bf16, expert e's LoRA_UP    (B_e = W_up)
 *   dW = sum_j (s * g_j) * B_{e_j} A_{e_j}
 *
 * Loops are written in the order of the definition: one output element at a
 * time, experts outermost, rank innermost.  The only concession to speed is an
 * OpenMP "parallel for" over independent output rows (no blocking, no
 * reordering of any sum).
 *
 * Pins (see tests/test_oracle_*.py): exhaustive bf16 round trip and exact
 * midpoint ties; exact rational brute force on tiny inputs; zero gates leave W
 * bit-identical; one expert with gate 1 equals a library fp64 GEMM; the merged
 * GEMV equals the dynamic-adapter output; permutation invariance; concat form
 * equals sum form; router closed forms (k = E full softmax, two-expert
 * sigmoid, shift invariance, argsort).  No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG 1

/* ------------------------------------------------------------------ bf16 */

/* bf16 is the upper 16 bits of an IEEE-754 binary32. */
double oracle_bf16_to_f64(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/*
 * Round a double to the nearest bf16 (ties to even) in ONE rounding step.
 * bf16 has 8 significant bits and binary32's exponent range, so a value with
 * binary exponent e (clamped to the subnormal exponent -126) lies on a grid of
 * spacing q = 2^(e-7).  x/q is exact (power-of-two scaling), nearbyint rounds
 * it to an integer with ties to even under the default rounding mode, and
 * n*q is exactly representable as a bf16 or rounds up to the next binade,
 * which is also on the grid.  Values at or beyond 2^128 become infinity.
 */
uint16_t oracle_f64_to_bf16_rne(double x)
{
    if (isnan(x)) return 0x7fc0;
    if (isinf(x)) return x > 0 ? 0x7f80 : 0xff80;
    if (x == 0.0) return signbit(x) ? 0x8000 : 0x0000;
    int e;
    (void)frexp(fabs(x), &e); /* |x| = m * 2^e, m in [0.5,1) -> exponent e-1 */
    int ex = e - 1;
    if (ex < -126) ex = -126;
    double q = ldexp(1.0, ex - 7);
    double n = nearbyint(x / q);
    double y = n * q;
    if (fabs(y) >= ldexp(1.0, 128)) return x > 0 ? 0x7f80 : 0xff80;
    float f = (float)y; /* exact: y has at most 8 significant bits */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(u >> 16);
}

/* Element-wise forms of the two conversions above, for array callers. */
void oracle_f64_to_bf16_rne_array(const double *x, uint16_t *y, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) y[i] = oracle_f64_to_bf16_rne(x[i]);
}

void oracle_bf16_to_f64_array(const uint16_t *x, double *y, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) y[i] = oracle_bf16_to_f64(x[i]);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------- router */

/*
 * Token-level pre-gating router (Eq.1's G(x) = Softmax(TopK(W_g x)), used once
 * per token as G^1(x^1), section "Model Structure").
 *
 *   hidden   [T][d] bf16      w_router [E][d] bf16 (no bias)
 *   logits   [T][E] fp64      l_e = sum_i h_i * W_r[e][i], i ascending
 *   logits32 [T][E] fp32      (float)l_e -- the precision the selection and the
 *                             gates are taken in (the kernel emits fp32 logits)
 *   idx      [T][k] int32     the k largest fp32 logits, ordered by
 *                             (logit descending, index ascending)
 *   gates    [T][k] fp64, gates32 = (float)gates
 *   gate_norm 0: softmax over the k selected logits (Eq.1; gates sum to 1)
 *   gate_norm 1: softmax over all E logits, then keep the k selected entries
 *                (the wording of "Router Architecture"; gates sum to < 1)
 * Any output pointer may be NULL.
 */
int oracle_pregate(const uint16_t *hidden, const uint16_t *w_router,
                   int T, int d, int E, int k, int gate_norm,
                   double *logits, float *logits32,
                   int32_t *idx, double *gates, float *gates32)
{
    if (!hidden || !w_router || T < 0 || d <= 0 || E <= 0 || k <= 0 || k > E ||
        (gate_norm != 0 && gate_norm != 1))
        return ORACLE_ERR_ARG;
    double *l = (double *)malloc(sizeof(double) * (size_t)E);
    float *lf = (float *)malloc(sizeof(float) * (size_t)E);
    char *taken = (char *)malloc((size_t)E);
    int *sel = (int *)malloc(sizeof(int) * (size_t)k);
    if (!l || !lf || !taken || !sel) { free(l); free(lf); free(taken); free(sel); return ORACLE_ERR_ARG; }

    for (int t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            double s = 0.0;
            for (int i = 0; i < d; ++i)
                s += oracle_bf16_to_f64(hidden[(size_t)t * d + i]) *
                     oracle_bf16_to_f64(w_router[(size_t)e * d + i]);
            l[e] = s;
            lf[e] = (float)s;
            taken[e] = 0;
            if (logits) logits[(size_t)t * E + e] = s;
            if (logits32) logits32[(size_t)t * E + e] = lf[e];
        }
        /* k rounds of arg-max; strict '>' keeps the lowest index among equals */
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || lf[e] > lf[best]) best = e;
            }
            taken[best] = 1;
            sel[j] = best;
            if (idx) idx[(size_t)t * k + j] = best;
        }
        /* softmax, max-subtracted, in fp64 from the fp32 logits */
        double m = (double)lf[sel[0]]; /* the overall maximum is selected first */
        double denom = 0.0;
        if (gate_norm == 0) {
            for (int j = 0; j < k; ++j) denom += exp((double)lf[sel[j]] - m);
        } else {
            for (int e = 0; e < E; ++e) denom += exp((double)lf[e] - m);
        }
        for (int j = 0; j < k; ++j) {
            double g = exp((double)lf[sel[j]] - m) / denom;
            if (gates) gates[(size_t)t * k + j] = g;
            if (gates32) gates32[(size_t)t * k + j] = (float)g;
        }
    }
    free(l); free(lf); free(taken); free(sel);
    return ORACLE_OK;
}

/* ---------------------------------------------------------------- switch */

/* dW[o][i] = sum_j (s*g_j) * sum_rho B_{e_j}[o][rho] * A_{e_j}[rho][i]  (Eq.4-6) */
static double delta_elem(const uint16_t *a_bank, const uint16_t *b_bank,
                         int out, int in, int r,
                         const int32_t *idx, const float *gates, int k,
                         float scale, int o, int i)
{
    double delta = 0.0;
    for (int j = 0; j < k; ++j) {
        const uint16_t *A = a_bank + (size_t)idx[j] * r * in;   /* [r][in]  */
        const uint16_t *B = b_bank + (size_t)idx[j] * out * r;  /* [out][r] */
        double p = 0.0;
        for (int rho = 0; rho < r; ++rho)
            p += oracle_bf16_to_f64(B[(size_t)o * r + rho]) *
                 oracle_bf16_to_f64(A[(size_t)rho * in + i]);
        delta += ((double)scale * (double)gates[j]) * p;
    }
    return delta;
}

static int check_switch_args(const void *w, const void *a, const void *b,
                             int out, int in, int64_t ldw, int E, int r,
                             const int32_t *idx, const float *gates, int k,
                             int row_begin, int row_end)
{
    if (!w || out <= 0 || in <= 0 || ldw < in || E <= 0 || r <= 0 || k < 0 ||
        row_begin < 0 || row_end > out || row_begin > row_end)
        return ORACLE_ERR_ARG;
    if (k > 0 && (!a || !b || !idx || !gates)) return ORACLE_ERR_ARG;
    for (int j = 0; j < k; ++j)
        if (idx[j] < 0 || idx[j] >= E) return ORACLE_ERR_ARG;
    return ORACLE_OK;
}

/*
 * Merged weight of one adapted matrix, rows [row_begin,row_end):
 *   W'[o][i] = bf16_rne( W_base[o][i] + dW[o][i] )          (Eq.6 / Eq.3)
 * computed in fp64 from the stored bits and rounded fp64 -> bf16 directly.
 * w_out is [row_end-row_begin][ld_out] bf16.  k = 0 gives W_base back.
 * This is also what the fused switch of Eq.8 yields in exact arithmetic: the
 * previous token's update cancels (W_{t-1} - dW_{t-1} + dW_t = W_base + dW_t).
 */
int oracle_merge_rows(const uint16_t *w_base, int64_t ldw,
                      const uint16_t *a_bank, const uint16_t *b_bank,
                      int out, int in, int E, int r,
                      const int32_t *idx, const float *gates, int k, float scale,
                      int row_begin, int row_end,
                      uint16_t *w_out, int64_t ld_out)
{
    int rc = check_switch_args(w_base, a_bank, b_bank, out, in, ldw, E, r, idx, gates, k, row_begin, row_end);
    if (rc || !w_out || ld_out < in) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int o = row_begin; o < row_end; ++o) {
        for (int i = 0; i < in; ++i) {
            double v = oracle_bf16_to_f64(w_base[(size_t)o * ldw + i]) +
                       delta_elem(a_bank, b_bank, out, in, r, idx, gates, k, scale, o, i);
            w_out[(size_t)(o - row_begin) * ld_out + i] = oracle_f64_to_bf16_rne(v);
        }
    }
    return ORACLE_OK;
}

/* Same as oracle_merge_rows but returns the un-rounded fp64 values W + dW. */
int oracle_merge_rows_f64(const uint16_t *w_base, int64_t ldw,
                          const uint16_t *a_bank, const uint16_t *b_bank,
                          int out, int in, int E, int r,
                          const int32_t *idx, const float *gates, int k, float scale,
                          int row_begin, int row_end,
                          double *w_out, int64_t ld_out)
{
    int rc = check_switch_args(w_base, a_bank, b_bank, out, in, ldw, E, r, idx, gates, k, row_begin, row_end);
    if (rc || !w_out || ld_out < in) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int o = row_begin; o < row_end; ++o)
        for (int i = 0; i < in; ++i)
            w_out[(size_t)(o - row_begin) * ld_out + i] =
                oracle_bf16_to_f64(w_base[(size_t)o * ldw + i]) +
                delta_elem(a_bank, b_bank, out, in, r, idx, gates, k, scale, o, i);
    return ORACLE_OK;
}

/*
 * Paper-literal in-place switch step (Eq.7-8): the matrix currently holds the
 * previous token's merge; subtract it and add the next token's in one update
 * with one rounding:
 *   W[o][i] <- bf16_rne( W_cur[o][i] + dW_next[o][i] - dW_prev[o][i] ).
 * The signed concatenation [-DOWN^{t-1}, DOWN^t] is taken term by term in that
 * order (previous experts first).
 */
int oracle_inplace_swap_rows(const uint16_t *w_cur, int64_t ldw,
                             const uint16_t *a_bank, const uint16_t *b_bank,
                             int out, int in, int E, int r,
                             const int32_t *idx_prev, const float *gates_prev, int k_prev,
                             const int32_t *idx_next, const float *gates_next, int k_next,
                             float scale, int row_begin, int row_end,
                             uint16_t *w_out, int64_t ld_out)
{
    int rc = check_switch_args(w_cur, a_bank, b_bank, out, in, ldw, E, r, idx_prev, gates_prev, k_prev, row_begin, row_end);
    if (rc) return rc;
    rc = check_switch_args(w_cur, a_bank, b_bank, out, in, ldw, E, r, idx_next, gates_next, k_next, row_begin, row_end);
    if (rc || !w_out || ld_out < in) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int o = row_begin; o < row_end; ++o) {
        for (int i = 0; i < in; ++i) {
            double v = oracle_bf16_to_f64(w_cur[(size_t)o * ldw + i]);
            v += -delta_elem(a_bank, b_bank, out, in, r, idx_prev, gates_prev, k_prev, scale, o, i) +
                 delta_elem(a_bank, b_bank, out, in, r, idx_next, gates_next, k_next, scale, o, i);
            w_out[(size_t)(o - row_begin) * ld_out + i] = oracle_f64_to_bf16_rne(v);
        }
    }
    return ORACLE_OK;
}

/*
 * The un-merged dynamic-adapter forward of one linear layer for one token
 * (Eq.1 / Eq.2 with the pre-gated weights):
 *   y = W_base x + s * sum_j g_j * B_{e_j} (A_{e_j} x)
 * x [in] fp64, y [out] fp64.  The adapter is applied as two mat-vecs, down
 * projection first, exactly as a dynamic adapter would run it.
 */
int oracle_dynamic_adapter_forward(const uint16_t *w_base, int64_t ldw,
                                   const uint16_t *a_bank, const uint16_t *b_bank,
                                   int out, int in, int E, int r,
                                   const int32_t *idx, const float *gates, int k, float scale,
                                   const double *x, double *y)
{
    int rc = check_switch_args(w_base, a_bank, b_bank, out, in, ldw, E, r, idx, gates, k, 0, out);
    if (rc || !x || !y) return ORACLE_ERR_ARG;
    double *z = (double *)malloc(sizeof(double) * (size_t)(k > 0 ? k : 1) * (size_t)r);
    if (!z) return ORACLE_ERR_ARG;
    for (int j = 0; j < k; ++j) {
        const uint16_t *A = a_bank + (size_t)idx[j] * r * in;
        for (int rho = 0; rho < r; ++rho) {
            double s = 0.0;
            for (int i = 0; i < in; ++i) s += oracle_bf16_to_f64(A[(size_t)rho * in + i]) * x[i];
            z[(size_t)j * r + rho] = s;
        }
    }
    for (int o = 0; o < out; ++o) {
        double base = 0.0;
        for (int i = 0; i < in; ++i) base += oracle_bf16_to_f64(w_base[(size_t)o * ldw + i]) * x[i];
        double ad = 0.0;
        for (int j = 0; j < k; ++j) {
            const uint16_t *B = b_bank + (size_t)idx[j] * out * r;
            double e = 0.0;
            for (int rho = 0; rho < r; ++rho) e += oracle_bf16_to_f64(B[(size_t)o * r + rho]) * z[(size_t)j * r + rho];
            ad += (double)gates[j] * e;
        }
        y[o] = base + (double)scale * ad;
    }
    free(z);
    return ORACLE_OK;
}

/* y = W x for a bf16 matrix and fp64 vector (the merged backbone's Eq.3). */
int oracle_gemv_bf16(const uint16_t *w, int64_t ldw, int out, int in, const double *x, double *y)
{
    if (!w || !x || !y || out <= 0 || in <= 0 || ldw < in) return ORACLE_ERR_ARG;
    for (int o = 0; o < out; ++o) {
        double s = 0.0;
        for (int i = 0; i < in; ++i) s += oracle_bf16_to_f64(w[(size_t)o * ldw + i]) * x[i];
        y[o] = s;
    }
    return ORACLE_OK;
}

/*
 * Distance in units of bf16 spacing between two bit patterns, on the monotone
 * integer line (sign-magnitude folded so that -0 and +0 coincide).  Writes the
 * maximum distance and the number of differing elements over n entries.
 */
int oracle_bf16_ulp_diff(const uint16_t *a, const uint16_t *b, int64_t n,
                         int64_t *max_ulp, int64_t *n_diff)
{
    if (!a || !b || n < 0) return ORACLE_ERR_ARG;
    int64_t mx = 0, nd = 0;
    for (int64_t i = 0; i < n; ++i) {
        int32_t x = (a[i] & 0x8000) ? -(int32_t)(a[i] & 0x7fff) : (int32_t)a[i];
        int32_t y = (b[i] & 0x8000) ? -(int32_t)(b[i] & 0x7fff) : (int32_t)b[i];
        int64_t dd = x > y ? (int64_t)x - y : (int64_t)y - x;
        if (dd) ++nd;
        if (dd > mx) mx = dd;
    }
    if (max_ulp) *max_ulp = mx;
    if (n_diff) *n_diff = nd;
    return ORACLE_OK;
}
