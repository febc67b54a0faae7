/*
 * CPU oracle for the mHC-lite hyper-connection path (and the Sinkhorn-Knopp
 * mHC variant it is compared with).  TEST INFRASTRUCTURE ONLY: a plain, slow,
 * fp64 transcription of the paper's definitions, used to check the GPU
 * library.  It shares no code, header, table or constant with the GPU path
 * and nothing in the product may call it.
 *
 * What each function follows:
 *   permutation table / P_stack ......... Theorem 3.1 (Birkhoff-von Neumann),
 *                                         Sec. 3.2 last paragraphs ("constant
 *                                         0/1 matrix in R^{n! x n^2}")
 *   coefficients, permutation form ...... Sec. 3.2, Eqs. (4)-(5) and the three
 *                                         unnumbered lines above them
 *   coefficients, Sinkhorn-Knopp form ... Sec. 2, Eq. (2) and the three lines
 *                                         above it; SK as described in Sec. 1
 *                                         and below Eq. (2) (20 repetitions)
 *   coefficients, permutation subset .... Sec. 5, paragraph on larger n
 *   stream mixing ........................ Sec. 2, Eq. (1)
 *   l1 error, relative range ............. Sec. 3.1, footnote 1 and Eq. (3)
 *   column sums, product over layers ..... Sec. 3.1 last paragraph, Sec. 4.3
 *   backward ............................. not in the paper: chain rule applied
 *                                         to the forward definitions above
 *
 * Readings taken where the paper is silent (the same ones the GPU library
 * documents): RMSNorm has no learnable gain and eps is added to the mean
 * square inside the root; x in R^{n x C} is flattened row-major; W is one
 * [nC, M] matrix with columns [res | pre | post]; permutations are in
 * lexicographic order with P_k[i][sigma_k(i)] = 1; H_post f is the outer
 * product; one SK iteration normalises columns, then rows.
 *
 * Pins (tests/test_oracle_*.py): brute-force permutation set, Birkhoff
 * invariants, one-hot / uniform / n=1 / n=2 closed forms, the closed form at
 * the paper's initialisation, an independent library implementation of the
 * forward, the paper's 3x3 SK example, central finite differences and a
 * library autograd for every backward; for the diagnostics, composition of
 * permutations, scaled doubly stochastic chains in closed form, a library
 * matrix product and the printed column sums of the 3x3 example; for the
 * permutation subset, bitwise equality with the full form when all n! are
 * given, circulant closed form, single-permutation and one-hot cases, finite
 * differences.  No function here is unpinned.
 *
 * All arrays are dense row-major doubles.  Tokens are independent; loops over
 * tokens are OpenMP-parallel, every sum inside a token and every sum over
 * tokens runs in plain index order.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#define MAXN 8
#define MAXF 40320 /* 8! */

int mhclo_factorial(int n)
{
    int f = 1;
    for (int i = 2; i <= n; ++i) f *= i;
    return f;
}

/* sigma[k][i], k = 0..n!-1 in lexicographic order of the tuples
 * (sigma(0), ..., sigma(n-1)); k = 0 is the identity. */
void mhclo_perm_table(int n, int *sigma)
{
    int cur[MAXN];
    for (int i = 0; i < n; ++i) cur[i] = i;
    int nf = mhclo_factorial(n);
    for (int k = 0; k < nf; ++k) {
        for (int i = 0; i < n; ++i) sigma[k * n + i] = cur[i];
        /* step to the lexicographic successor */
        int p = n - 2;
        while (p >= 0 && cur[p] > cur[p + 1]) --p;
        if (p < 0) break;
        int q = n - 1;
        while (cur[q] < cur[p]) --q;
        int tmp = cur[p]; cur[p] = cur[q]; cur[q] = tmp;
        for (int lo = p + 1, hi = n - 1; lo < hi; ++lo, --hi) {
            tmp = cur[lo]; cur[lo] = cur[hi]; cur[hi] = tmp;
        }
    }
}

/* P[k][i][j] = 1 if sigma_k(i) == j else 0: the concatenation of all n!
 * permutation matrices (Sec. 3.2). */
void mhclo_pstack(int n, double *P)
{
    int nf = mhclo_factorial(n);
    int *sigma = (int *)malloc(sizeof(int) * (size_t)nf * n);
    mhclo_perm_table(n, sigma);
    memset(P, 0, sizeof(double) * (size_t)nf * n * n);
    for (int k = 0; k < nf; ++k)
        for (int i = 0; i < n; ++i)
            P[((size_t)k * n + i) * n + sigma[k * n + i]] = 1.0;
    free(sigma);
}

/* x_hat' = RMSNorm(x_hat), u = x_hat' W, z = alpha_g u + b   (one token).
 * Normalises first and multiplies afterwards, exactly as written. */
static void token_logits(int nC, int M, int R, int n, const double *xh, const double *W,
                         const double *b, const double *alpha, double eps,
                         double *xn, double *r_out, double *u, double *z)
{
    double ss = 0.0;
    for (int k = 0; k < nC; ++k) ss += xh[k] * xh[k];
    double r = 1.0 / sqrt(ss / (double)nC + eps);
    for (int k = 0; k < nC; ++k) xn[k] = xh[k] * r;
    for (int m = 0; m < M; ++m) {
        double acc = 0.0;
        for (int k = 0; k < nC; ++k) acc += xn[k] * W[(size_t)k * M + m];
        u[m] = acc;
    }
    for (int m = 0; m < M; ++m) {
        int g = (m < R) ? 0 : (m < R + n ? 1 : 2);
        z[m] = alpha[g] * u[m] + b[m];
    }
    *r_out = r;
}

static double sigmoid(double t) { return 1.0 / (1.0 + exp(-t)); }

static void softmax(int R, const double *z, double *a)
{
    double zmax = z[0];
    for (int k = 1; k < R; ++k) if (z[k] > zmax) zmax = z[k];
    double s = 0.0;
    for (int k = 0; k < R; ++k) { a[k] = exp(z[k] - zmax); s += a[k]; }
    for (int k = 0; k < R; ++k) a[k] /= s;
}

/* Sec. 3.2: H_pre = sigmoid(.), H_post = 2 sigmoid(.), a = softmax(.),
 * H_res = sum_k a_k P_k (dense contraction with the 0/1 stack P [R][n][n]).
 * a_out (nullable) receives the weights a, [T][R]. */
static void coeffs_stack(int n, int C, long T, int R, const double *P, const double *x,
                         const double *W, const double *b, const double *alpha, double eps,
                         double *H_res, double *H_pre, double *H_post, double *a_out)
{
    int nC = n * C, M = R + 2 * n;
#pragma omp parallel
    {
        double *xn = (double *)malloc(sizeof(double) * nC);
        double *u = (double *)malloc(sizeof(double) * M);
        double *z = (double *)malloc(sizeof(double) * M);
        double *a = (double *)malloc(sizeof(double) * R);
#pragma omp for schedule(static)
        for (long t = 0; t < T; ++t) {
            double r;
            token_logits(nC, M, R, n, x + (size_t)t * nC, W, b, alpha, eps, xn, &r, u, z);
            softmax(R, z, a);
            for (int i = 0; i < n; ++i)
                for (int j = 0; j < n; ++j) {
                    double acc = 0.0;
                    for (int k = 0; k < R; ++k) acc += a[k] * P[((size_t)k * n + i) * n + j];
                    H_res[((size_t)t * n + i) * n + j] = acc;
                }
            for (int j = 0; j < n; ++j) {
                H_pre[(size_t)t * n + j] = sigmoid(z[R + j]);
                H_post[(size_t)t * n + j] = 2.0 * sigmoid(z[R + n + j]);
            }
            if (a_out) for (int k = 0; k < R; ++k) a_out[(size_t)t * R + k] = a[k];
        }
        free(xn); free(u); free(z); free(a);
    }
}

/* All n! permutations, lexicographic order (Sec. 3.2, Eqs. (4)-(5)). */
void mhclo_coeffs_lite(int n, int C, long T, const double *x, const double *W, const double *b,
                       const double *alpha, double eps,
                       double *H_res, double *H_pre, double *H_post, double *a_out)
{
    int R = mhclo_factorial(n);
    double *P = (double *)malloc(sizeof(double) * (size_t)R * n * n);
    mhclo_pstack(n, P);
    coeffs_stack(n, C, T, R, P, x, W, b, alpha, eps, H_res, H_pre, H_post, a_out);
    free(P);
}

/* P[k][i][j] = 1 if sigma[k][i] == j for K given permutations. */
static double *stack_of(int n, int K, const int *sigma)
{
    double *P = (double *)calloc((size_t)K * n * n, sizeof(double));
    for (int k = 0; k < K; ++k)
        for (int i = 0; i < n; ++i) P[((size_t)k * n + i) * n + sigma[k * n + i]] = 1.0;
    return P;
}

/* The same with only K chosen permutations sigma [K][n] (Sec. 5, discussion
 * of larger n: a subset of the permutation matrices; the result stays doubly
 * stochastic).  Logit columns [K | n | n]. */
void mhclo_coeffs_subset(int n, int C, long T, int K, const int *sigma, const double *x,
                         const double *W, const double *b, const double *alpha, double eps,
                         double *H_res, double *H_pre, double *H_post, double *a_out)
{
    double *P = stack_of(n, K, sigma);
    coeffs_stack(n, C, T, K, P, x, W, b, alpha, eps, H_res, H_pre, H_post, a_out);
    free(P);
}

/* Sinkhorn-Knopp on one n x n matrix: `iters` times (all columns rescaled to
 * sum 1, then all rows rescaled to sum 1).  If `trace` is non-null it receives
 * the matrix after every half step, [2*iters][n][n], and `sums` the divisors,
 * [2*iters][n]. */
static void sk_run(int n, const double *X0, int iters, double *X, double *trace, double *sums)
{
    for (int e = 0; e < n * n; ++e) X[e] = X0[e];
    for (int it = 0; it < iters; ++it) {
        for (int j = 0; j < n; ++j) {
            double s = 0.0;
            for (int i = 0; i < n; ++i) s += X[i * n + j];
            for (int i = 0; i < n; ++i) X[i * n + j] /= s;
            if (sums) sums[(2 * it) * n + j] = s;
        }
        if (trace) memcpy(trace + (size_t)(2 * it) * n * n, X, sizeof(double) * n * n);
        for (int i = 0; i < n; ++i) {
            double s = 0.0;
            for (int j = 0; j < n; ++j) s += X[i * n + j];
            for (int j = 0; j < n; ++j) X[i * n + j] /= s;
            if (sums) sums[(2 * it + 1) * n + i] = s;
        }
        if (trace) memcpy(trace + (size_t)(2 * it + 1) * n * n, X, sizeof(double) * n * n);
    }
}

void mhclo_sk(int n, const double *X0, int iters, double *X)
{
    sk_run(n, X0, iters, X, NULL, NULL);
}

/* Sec. 2, Eq. (2): H_res = SK(exp(mat(alpha_res x_hat' W_res + b_res))), the
 * gates as in the permutation form.  M = n^2 + 2n. */
void mhclo_coeffs_sk(int n, int C, long T, const double *x, const double *W, const double *b,
                     const double *alpha, double eps, int iters,
                     double *H_res, double *H_pre, double *H_post)
{
    int nC = n * C, R = n * n, M = R + 2 * n;
#pragma omp parallel
    {
        double *xn = (double *)malloc(sizeof(double) * nC);
        double *u = (double *)malloc(sizeof(double) * M);
        double *z = (double *)malloc(sizeof(double) * M);
        double E[MAXN * MAXN];
#pragma omp for schedule(static)
        for (long t = 0; t < T; ++t) {
            double r;
            token_logits(nC, M, R, n, x + (size_t)t * nC, W, b, alpha, eps, xn, &r, u, z);
            for (int e = 0; e < R; ++e) E[e] = exp(z[e]);
            sk_run(n, E, iters, H_res + (size_t)t * R, NULL, NULL);
            for (int j = 0; j < n; ++j) {
                H_pre[(size_t)t * n + j] = sigmoid(z[R + j]);
                H_post[(size_t)t * n + j] = 2.0 * sigmoid(z[R + n + j]);
            }
        }
        free(xn); free(u); free(z);
    }
}

/* Eq. (1), inner part: h = H_pre x  (a 1 x n row times the n x C streams). */
void mhclo_pre(int n, int C, long T, const double *x, const double *H_pre, double *h)
{
#pragma omp parallel for schedule(static)
    for (long t = 0; t < T; ++t)
        for (int c = 0; c < C; ++c) {
            double acc = 0.0;
            for (int j = 0; j < n; ++j)
                acc += H_pre[(size_t)t * n + j] * x[((size_t)t * n + j) * C + c];
            h[(size_t)t * C + c] = acc;
        }
}

/* Eq. (1): x_out = H_res x + H_post^T y, with y = f(H_pre x) supplied. */
void mhclo_post(int n, int C, long T, const double *x, const double *y, const double *H_res,
                const double *H_post, double *x_out)
{
#pragma omp parallel for schedule(static)
    for (long t = 0; t < T; ++t)
        for (int i = 0; i < n; ++i)
            for (int c = 0; c < C; ++c) {
                double acc = 0.0;
                for (int j = 0; j < n; ++j)
                    acc += H_res[((size_t)t * n + i) * n + j] * x[((size_t)t * n + j) * C + c];
                acc += H_post[(size_t)t * n + i] * y[(size_t)t * C + c];
                x_out[((size_t)t * n + i) * C + c] = acc;
            }
}

/* Backward of mhclo_post with x, y, H_res, H_post independent inputs.
 * g_x is overwritten with the part of dL/dx that flows through H_res x. */
void mhclo_post_bwd(int n, int C, long T, const double *x, const double *y, const double *H_res,
                    const double *H_post, const double *g_xout,
                    double *g_x, double *g_y, double *g_H_res, double *g_H_post)
{
#pragma omp parallel for schedule(static)
    for (long t = 0; t < T; ++t) {
        const double *xt = x + (size_t)t * n * C, *gt = g_xout + (size_t)t * n * C;
        const double *yt = y + (size_t)t * C;
        for (int c = 0; c < C; ++c) {
            double acc = 0.0;
            for (int i = 0; i < n; ++i) acc += H_post[(size_t)t * n + i] * gt[(size_t)i * C + c];
            g_y[(size_t)t * C + c] = acc;
        }
        for (int i = 0; i < n; ++i) {
            double acc = 0.0;
            for (int c = 0; c < C; ++c) acc += gt[(size_t)i * C + c] * yt[c];
            g_H_post[(size_t)t * n + i] = acc;
            for (int j = 0; j < n; ++j) {
                double d = 0.0;
                for (int c = 0; c < C; ++c) d += gt[(size_t)i * C + c] * xt[(size_t)j * C + c];
                g_H_res[((size_t)t * n + i) * n + j] = d;
            }
        }
        for (int j = 0; j < n; ++j)
            for (int c = 0; c < C; ++c) {
                double acc = 0.0;
                for (int i = 0; i < n; ++i)
                    acc += H_res[((size_t)t * n + i) * n + j] * gt[(size_t)i * C + c];
                g_x[((size_t)t * n + j) * C + c] = acc;
            }
    }
}

/* Backward of mhclo_pre.  g_x is accumulated into (+=). */
void mhclo_pre_bwd(int n, int C, long T, const double *x, const double *H_pre, const double *g_h,
                   double *g_x, double *g_H_pre)
{
#pragma omp parallel for schedule(static)
    for (long t = 0; t < T; ++t)
        for (int j = 0; j < n; ++j) {
            double acc = 0.0;
            for (int c = 0; c < C; ++c) {
                acc += g_h[(size_t)t * C + c] * x[((size_t)t * n + j) * C + c];
                g_x[((size_t)t * n + j) * C + c] += H_pre[(size_t)t * n + j] * g_h[(size_t)t * C + c];
            }
            g_H_pre[(size_t)t * n + j] = acc;
        }
}

/* Shared tail of both coefficient backwards: from per-token g_z (gradient on
 * the logits z, [T][M]) and the recomputed r, u accumulate g_b, g_alpha, g_W
 * and add the RMSNorm/projection part to g_x.
 *   z_m = alpha_g u_m + b_m, u = x_hat' W, x_hat' = r x_hat,
 *   r = (mean(x_hat^2) + eps)^(-1/2). */
static void logits_bwd(int n, int C, long T, int R, const double *x, const double *W,
                       const double *alpha, double eps, const double *g_z /*[T][M]*/,
                       double *g_x, double *g_W, double *g_b, double *g_alpha)
{
    int nC = n * C, M = R + 2 * n;
    double *v = (double *)malloc(sizeof(double) * (size_t)T * M);   /* alpha_g g_z */
    double *rr = (double *)malloc(sizeof(double) * (size_t)T);
    double *uu = (double *)malloc(sizeof(double) * (size_t)T * M);
#pragma omp parallel
    {
        double *xn = (double *)malloc(sizeof(double) * nC);
        double *gxn = (double *)malloc(sizeof(double) * nC);
#pragma omp for schedule(static)
        for (long t = 0; t < T; ++t) {
            const double *xh = x + (size_t)t * nC;
            double ss = 0.0;
            for (int k = 0; k < nC; ++k) ss += xh[k] * xh[k];
            double r = 1.0 / sqrt(ss / (double)nC + eps);
            rr[t] = r;
            for (int k = 0; k < nC; ++k) xn[k] = xh[k] * r;
            for (int m = 0; m < M; ++m) {
                double acc = 0.0;
                for (int k = 0; k < nC; ++k) acc += xn[k] * W[(size_t)k * M + m];
                uu[(size_t)t * M + m] = acc;
                int g = (m < R) ? 0 : (m < R + n ? 1 : 2);
                v[(size_t)t * M + m] = alpha[g] * g_z[(size_t)t * M + m];
            }
            /* g on x_hat' = W v ; then through x_hat' = r x_hat */
            double dot = 0.0;
            for (int k = 0; k < nC; ++k) {
                double acc = 0.0;
                for (int m = 0; m < M; ++m) acc += W[(size_t)k * M + m] * v[(size_t)t * M + m];
                gxn[k] = acc;
                dot += acc * xh[k];
            }
            double coef = r * r * r / (double)nC * dot;
            for (int k = 0; k < nC; ++k) g_x[(size_t)t * nC + k] += r * gxn[k] - coef * xh[k];
        }
        free(xn); free(gxn);
    }
    for (int m = 0; m < M; ++m) g_b[m] = 0.0;
    for (int g = 0; g < 3; ++g) g_alpha[g] = 0.0;
    for (long t = 0; t < T; ++t)
        for (int m = 0; m < M; ++m) {
            int g = (m < R) ? 0 : (m < R + n ? 1 : 2);
            g_b[m] += g_z[(size_t)t * M + m];
            g_alpha[g] += g_z[(size_t)t * M + m] * uu[(size_t)t * M + m];
        }
    /* g_W[k][m] = sum_t x_hat'_t[k] v_t[m], tokens in order */
#pragma omp parallel for schedule(static)
    for (int k = 0; k < nC; ++k)
        for (int m = 0; m < M; ++m) {
            double acc = 0.0;
            for (long t = 0; t < T; ++t)
                acc += rr[t] * x[(size_t)t * nC + k] * v[(size_t)t * M + m];
            g_W[(size_t)k * M + m] = acc;
        }
    free(v); free(rr); free(uu);
}

/* Backward of coeffs_stack.  Recomputes the forward from x.  g_x is
 * accumulated into; g_W, g_b, g_alpha are overwritten. */
static void coeffs_stack_bwd(int n, int C, long T, int R, const double *P, const double *x,
                             const double *W, const double *b, const double *alpha, double eps,
                             const double *g_H_res, const double *g_H_pre, const double *g_H_post,
                             double *g_x, double *g_W, double *g_b, double *g_alpha)
{
    int nC = n * C, M = R + 2 * n;
    double *g_z = (double *)malloc(sizeof(double) * (size_t)T * M);
#pragma omp parallel
    {
        double *xn = (double *)malloc(sizeof(double) * nC);
        double *u = (double *)malloc(sizeof(double) * M);
        double *z = (double *)malloc(sizeof(double) * M);
        double *a = (double *)malloc(sizeof(double) * R);
        double *g_a = (double *)malloc(sizeof(double) * R);
#pragma omp for schedule(static)
        for (long t = 0; t < T; ++t) {
            double r;
            token_logits(nC, M, R, n, x + (size_t)t * nC, W, b, alpha, eps, xn, &r, u, z);
            softmax(R, z, a);
            /* H_res = sum_k a_k P_k  =>  g_a[k] = <g_H_res, P_k> */
            double mean = 0.0;
            for (int k = 0; k < R; ++k) {
                double acc = 0.0;
                for (int i = 0; i < n; ++i)
                    for (int j = 0; j < n; ++j)
                        acc += g_H_res[((size_t)t * n + i) * n + j] * P[((size_t)k * n + i) * n + j];
                g_a[k] = acc;
                mean += a[k] * acc;
            }
            for (int k = 0; k < R; ++k) g_z[(size_t)t * M + k] = a[k] * (g_a[k] - mean);
            for (int j = 0; j < n; ++j) {
                double sp = sigmoid(z[R + j]), sq = sigmoid(z[R + n + j]);
                g_z[(size_t)t * M + R + j] = g_H_pre[(size_t)t * n + j] * sp * (1.0 - sp);
                g_z[(size_t)t * M + R + n + j] = g_H_post[(size_t)t * n + j] * 2.0 * sq * (1.0 - sq);
            }
        }
        free(xn); free(u); free(z); free(a); free(g_a);
    }
    logits_bwd(n, C, T, R, x, W, alpha, eps, g_z, g_x, g_W, g_b, g_alpha);
    free(g_z);
}

void mhclo_coeffs_lite_bwd(int n, int C, long T, const double *x, const double *W, const double *b,
                           const double *alpha, double eps,
                           const double *g_H_res, const double *g_H_pre, const double *g_H_post,
                           double *g_x, double *g_W, double *g_b, double *g_alpha)
{
    int R = mhclo_factorial(n);
    double *P = (double *)malloc(sizeof(double) * (size_t)R * n * n);
    mhclo_pstack(n, P);
    coeffs_stack_bwd(n, C, T, R, P, x, W, b, alpha, eps, g_H_res, g_H_pre, g_H_post, g_x, g_W,
                     g_b, g_alpha);
    free(P);
}

void mhclo_coeffs_subset_bwd(int n, int C, long T, int K, const int *sigma, const double *x,
                             const double *W, const double *b, const double *alpha, double eps,
                             const double *g_H_res, const double *g_H_pre,
                             const double *g_H_post, double *g_x, double *g_W, double *g_b,
                             double *g_alpha)
{
    double *P = stack_of(n, K, sigma);
    coeffs_stack_bwd(n, C, T, K, P, x, W, b, alpha, eps, g_H_res, g_H_pre, g_H_post, g_x, g_W,
                     g_b, g_alpha);
    free(P);
}

/* Backward of mhclo_coeffs_sk: re-runs SK keeping every half step, then walks
 * the 2*iters normalisations in reverse.  For Y = X / s with s the column (or
 * row) sums: g_X = (g_Y - sum_along_axis(g_Y * Y)) / s. */
void mhclo_coeffs_sk_bwd(int n, int C, long T, const double *x, const double *W, const double *b,
                         const double *alpha, double eps, int iters,
                         const double *g_H_res, const double *g_H_pre, const double *g_H_post,
                         double *g_x, double *g_W, double *g_b, double *g_alpha)
{
    int nC = n * C, R = n * n, M = R + 2 * n;
    double *g_z = (double *)malloc(sizeof(double) * (size_t)T * M);
#pragma omp parallel
    {
        double *xn = (double *)malloc(sizeof(double) * nC);
        double *u = (double *)malloc(sizeof(double) * M);
        double *z = (double *)malloc(sizeof(double) * M);
        double *trace = (double *)malloc(sizeof(double) * (size_t)(2 * iters + 1) * R);
        double *sums = (double *)malloc(sizeof(double) * (size_t)(2 * iters + 1) * n);
        double E[MAXN * MAXN], Xf[MAXN * MAXN], g[MAXN * MAXN];
#pragma omp for schedule(static)
        for (long t = 0; t < T; ++t) {
            double r;
            token_logits(nC, M, R, n, x + (size_t)t * nC, W, b, alpha, eps, xn, &r, u, z);
            for (int e = 0; e < R; ++e) E[e] = exp(z[e]);
            sk_run(n, E, iters, Xf, trace, sums);
            for (int e = 0; e < R; ++e) g[e] = g_H_res[(size_t)t * R + e];
            for (int it = iters - 1; it >= 0; --it) {
                const double *Y = trace + (size_t)(2 * it + 1) * R;   /* after the row step */
                const double *s = sums + (size_t)(2 * it + 1) * n;
                for (int i = 0; i < n; ++i) {
                    double d = 0.0;
                    for (int j = 0; j < n; ++j) d += g[i * n + j] * Y[i * n + j];
                    for (int j = 0; j < n; ++j) g[i * n + j] = (g[i * n + j] - d) / s[i];
                }
                Y = trace + (size_t)(2 * it) * R;                    /* after the column step */
                s = sums + (size_t)(2 * it) * n;
                for (int j = 0; j < n; ++j) {
                    double d = 0.0;
                    for (int i = 0; i < n; ++i) d += g[i * n + j] * Y[i * n + j];
                    for (int i = 0; i < n; ++i) g[i * n + j] = (g[i * n + j] - d) / s[j];
                }
            }
            for (int e = 0; e < R; ++e) g_z[(size_t)t * M + e] = g[e] * E[e];
            for (int j = 0; j < n; ++j) {
                double sp = sigmoid(z[R + j]), sq = sigmoid(z[R + n + j]);
                g_z[(size_t)t * M + R + j] = g_H_pre[(size_t)t * n + j] * sp * (1.0 - sp);
                g_z[(size_t)t * M + R + n + j] = g_H_post[(size_t)t * n + j] * 2.0 * sq * (1.0 - sq);
            }
        }
        free(xn); free(u); free(z); free(trace); free(sums);
    }
    logits_bwd(n, C, T, R, x, W, alpha, eps, g_z, g_x, g_W, g_b, g_alpha);
    free(g_z);
}

/* Footnote 1 of Sec. 3.1: ||X 1 - 1||_1 + ||X^T 1 - 1||_1 for each of T
 * n x n matrices; and Eq. (3): nu = min positive entry / max entry. */
void mhclo_ds_l1_error(int n, long T, const double *X, double *err)
{
    for (long t = 0; t < T; ++t) {
        const double *Xt = X + (size_t)t * n * n;
        double e = 0.0;
        for (int i = 0; i < n; ++i) {
            double s = 0.0;
            for (int j = 0; j < n; ++j) s += Xt[i * n + j];
            e += fabs(s - 1.0);
        }
        for (int j = 0; j < n; ++j) {
            double s = 0.0;
            for (int i = 0; i < n; ++i) s += Xt[i * n + j];
            e += fabs(s - 1.0);
        }
        err[t] = e;
    }
}

void mhclo_relative_range(int n, long T, const double *X, double *nu)
{
    for (long t = 0; t < T; ++t) {
        const double *Xt = X + (size_t)t * n * n;
        double mx = Xt[0], mn = INFINITY;
        for (int e = 0; e < n * n; ++e) {
            if (Xt[e] > mx) mx = Xt[e];
            if (Xt[e] > 0.0 && Xt[e] < mn) mn = Xt[e];
        }
        nu[t] = mn / mx;
    }
}

/* The logits themselves (Sec. 3.2, the three lines above Eq. (4); Sec. 2 for
 * the Sinkhorn-Knopp form): z = alpha_g (RMSNorm(x_hat) W) + b for every
 * token, [T][M], R = number of residual logits (n! or n^2). */
void mhclo_logits(int n, int C, long T, int R, const double *x, const double *W, const double *b,
                  const double *alpha, double eps, double *z)
{
    int nC = n * C, M = R + 2 * n;
#pragma omp parallel
    {
        double *xn = (double *)malloc(sizeof(double) * nC);
        double *u = (double *)malloc(sizeof(double) * M);
#pragma omp for schedule(static)
        for (long t = 0; t < T; ++t) {
            double r;
            token_logits(nC, M, R, n, x + (size_t)t * nC, W, b, alpha, eps, xn, &r, u,
                         z + (size_t)t * M);
        }
        free(xn); free(u);
    }
}

/* Sec. 3.1 (accumulation over depth) and Sec. 4.3 (column sums of single
 * residual matrices and of their product over the layers): for L layers of
 * per-token matrices H[l][t] (n x n) this writes
 *   colsum[l][t][j]      = sum_i H[l][t][i][j]
 *   l1[l][t]             = l1 error of H[l][t]           (footnote 1 of Sec. 3.1)
 *   Q_l = H[l] Q_{l-1}, Q_0 = I   (the matrix that carries x_1 to x_{l+1} when
 *                                  only the residual term of Eq. (1) is kept)
 *   prod_colsum[l][t][j] = sum_i Q_l[i][j],   prod_l1[l][t] = l1 error of Q_l
 *   prod[t]              = Q_L
 * The paper does not say on which side later layers multiply; this takes the
 * order in which Eq. (1) applies them. */
void mhclo_ds_chain(int n, int L, long T, const double *H, double *colsum, double *l1,
                    double *prod, double *prod_colsum, double *prod_l1)
{
    int nn = n * n;
    for (long t = 0; t < T; ++t) {
        double Q[MAXN * MAXN], Qn[MAXN * MAXN];
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) Q[i * n + j] = (i == j) ? 1.0 : 0.0;
        for (int l = 0; l < L; ++l) {
            const double *Hl = H + ((size_t)l * T + t) * nn;
            for (int j = 0; j < n; ++j) {
                double s = 0.0;
                for (int i = 0; i < n; ++i) s += Hl[i * n + j];
                colsum[((size_t)l * T + t) * n + j] = s;
            }
            mhclo_ds_l1_error(n, 1, Hl, l1 + (size_t)l * T + t);
            for (int i = 0; i < n; ++i)
                for (int j = 0; j < n; ++j) {
                    double s = 0.0;
                    for (int k = 0; k < n; ++k) s += Hl[i * n + k] * Q[k * n + j];
                    Qn[i * n + j] = s;
                }
            memcpy(Q, Qn, sizeof(double) * nn);
            for (int j = 0; j < n; ++j) {
                double s = 0.0;
                for (int i = 0; i < n; ++i) s += Q[i * n + j];
                prod_colsum[((size_t)l * T + t) * n + j] = s;
            }
            mhclo_ds_l1_error(n, 1, Q, prod_l1 + (size_t)l * T + t);
        }
        memcpy(prod + (size_t)t * nn, Q, sizeof(double) * nn);
    }
}
