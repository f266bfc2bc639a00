/*
 * fp64 CPU oracle for the K-FAC work items (test infrastructure only).
 *
 * This file is the slow, plain reference that the GPU library is checked
 * against.  It is NOT part of the product path: only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may load it.  It shares
 * no code, headers, tables or helpers with the HIP sources.
 *
 * What it computes (PipeFisher, section 2.3.1 "Work in K-FAC"):
 *   - a Kronecker factor is the mini-batch mean of outer products of the
 *     per-example layer inputs (A) or output errors (B): U U^T with
 *     U = [a_1 ... a_n]/sqrt(n)                  -> oracle_curvature
 *   - each factor is symmetric, so its inverse is taken through a Cholesky
 *     decomposition followed by the inverse from the Cholesky factor
 *                                                -> oracle_invert
 *   - the preconditioned gradient is B^-1 G A^-1 -> oracle_precondition
 *   - the Kronecker identities (A (x) B)^-1 = A^-1 (x) B^-1 and
 *     (A (x) B) vec(X) = vec(B X A), vec stacking columns, are checked by
 *     forming the Kronecker product explicitly    -> oracle_kron_solve
 * The damping term (lambda added to each factor's diagonal before the
 * inversion) is not in the paper; it is this build's stated reading.
 *
 * All matrices are row-major double.  Every routine is the textbook loop
 * nest; OpenMP only distributes independent rows / right-hand sides.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* factor[i][j] = beta*factor[i][j] + alpha * sum_t x[t][i]*x[t][j]
 * x is n x d (row t = example t), factor is d x d.  With alpha = 1/n and
 * beta = 0 this is <a a^T> over the examples (section 2.3, definition of
 * A_l and B_l; section 2.3.1, A = U_A U_A^T). */
void oracle_curvature(const double *x, int64_t n, int64_t d, int64_t ldx,
                      double alpha, double beta, double *factor, int64_t ldf)
{
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < d; ++i) {
        double *row = (double *)calloc((size_t)d, sizeof(double));
        for (int64_t t = 0; t < n; ++t) {
            const double xi = x[t * ldx + i];
            const double *xt = x + t * ldx;
            for (int64_t j = 0; j < d; ++j) row[j] += xi * xt[j];
        }
        for (int64_t j = 0; j < d; ++j) {
            const double old = (beta == 0.0) ? 0.0 : beta * factor[i * ldf + j];
            factor[i * ldf + j] = old + alpha * row[j];
        }
        free(row);
    }
}

/* Cholesky decomposition m = l l^T, l lower triangular, column by column
 * (Cholesky-Crout).  m and l are d x d row-major; only the lower triangle of
 * m is read; the strict upper triangle of l is set to zero.
 * Returns 0, or k (1-based) if the k-th pivot is not positive / not finite. */
int64_t oracle_cholesky(const double *m, int64_t d, int64_t ldm, double *l, int64_t ldl)
{
    for (int64_t i = 0; i < d; ++i)
        for (int64_t j = 0; j < d; ++j) l[i * ldl + j] = 0.0;
    for (int64_t j = 0; j < d; ++j) {
        double s = m[j * ldm + j];
        for (int64_t k = 0; k < j; ++k) s -= l[j * ldl + k] * l[j * ldl + k];
        if (!(s > 0.0) || !isfinite(s)) return j + 1;
        const double ljj = sqrt(s);
        l[j * ldl + j] = ljj;
#pragma omp parallel for schedule(static)
        for (int64_t i = j + 1; i < d; ++i) {
            double t = m[i * ldm + j];
            const double *li = l + i * ldl, *lj = l + j * ldl;
            for (int64_t k = 0; k < j; ++k) t -= li[k] * lj[k];
            l[i * ldl + j] = t / ljj;
        }
    }
    return 0;
}

/* inv = (l l^T)^-1 from the Cholesky factor: solve l y = I by forward
 * substitution, then l^T x = y by back substitution, for all columns of the
 * identity.  Each thread owns a range of right-hand-side columns. */
void oracle_cholesky_inverse(const double *l, int64_t d, int64_t ldl, double *inv, int64_t ldi)
{
#pragma omp parallel
    {
        int nt = 1, id = 0;
#ifdef _OPENMP
        nt = omp_get_num_threads();
        id = omp_get_thread_num();
#endif
        const int64_t c0 = d * id / nt, c1 = d * (id + 1) / nt;
        /* forward: y[i][c] = (I[i][c] - sum_{k<i} l[i][k] y[k][c]) / l[i][i] */
        for (int64_t i = 0; i < d; ++i) {
            double *yi = inv + i * ldi;
            for (int64_t c = c0; c < c1; ++c) yi[c] = (c == i) ? 1.0 : 0.0;
            for (int64_t k = 0; k < i; ++k) {
                const double lik = l[i * ldl + k];
                const double *yk = inv + k * ldi;
                for (int64_t c = c0; c < c1; ++c) yi[c] -= lik * yk[c];
            }
            const double lii = l[i * ldl + i];
            for (int64_t c = c0; c < c1; ++c) yi[c] /= lii;
        }
        /* backward: x[i][c] = (y[i][c] - sum_{k>i} l[k][i] x[k][c]) / l[i][i] */
        for (int64_t i = d - 1; i >= 0; --i) {
            double *xi = inv + i * ldi;
            for (int64_t k = i + 1; k < d; ++k) {
                const double lki = l[k * ldl + i];
                const double *xk = inv + k * ldi;
                for (int64_t c = c0; c < c1; ++c) xi[c] -= lki * xk[c];
            }
            const double lii = l[i * ldl + i];
            for (int64_t c = c0; c < c1; ++c) xi[c] /= lii;
        }
    }
}

/* inv = (factor + damping*I)^-1 through Cholesky (section 2.3.1: Cholesky
 * decomposition followed by the inverse from it).  Returns the Cholesky
 * status; inv is untouched if the matrix is not positive definite. */
int64_t oracle_invert(const double *factor, int64_t d, int64_t ldf, double damping,
                      double *inv, int64_t ldi)
{
    double *m = (double *)malloc((size_t)d * d * sizeof(double));
    double *l = (double *)malloc((size_t)d * d * sizeof(double));
    for (int64_t i = 0; i < d; ++i)
        for (int64_t j = 0; j < d; ++j)
            m[i * d + j] = factor[i * ldf + j] + ((i == j) ? damping : 0.0);
    const int64_t info = oracle_cholesky(m, d, d, l, d);
    if (info == 0) oracle_cholesky_inverse(l, d, d, inv, ldi);
    free(m);
    free(l);
    return info;
}

/* out = b_inv * grad * a_inv; grad and out are d_out x d_in, b_inv is
 * d_out x d_out, a_inv is d_in x d_in (section 2.3.1, B^-1 G A^-1). */
void oracle_precondition(const double *b_inv, int64_t d_out, const double *a_inv, int64_t d_in,
                         const double *grad, double *out)
{
    double *t = (double *)malloc((size_t)d_out * d_in * sizeof(double));
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < d_out; ++i) {
        double *ti = t + i * d_in;
        for (int64_t j = 0; j < d_in; ++j) ti[j] = 0.0;
        for (int64_t k = 0; k < d_out; ++k) {
            const double b = b_inv[i * d_out + k];
            const double *gk = grad + k * d_in;
            for (int64_t j = 0; j < d_in; ++j) ti[j] += b * gk[j];
        }
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < d_out; ++i) {
        double *oi = out + i * d_in;
        const double *ti = t + i * d_in;
        for (int64_t j = 0; j < d_in; ++j) oi[j] = 0.0;
        for (int64_t k = 0; k < d_in; ++k) {
            const double tk = ti[k];
            const double *ak = a_inv + k * d_in;
            for (int64_t j = 0; j < d_in; ++j) oi[j] += tk * ak[j];
        }
    }
    free(t);
}

/* Brute force for tiny layers: form K = (A + damping I) (x) (B + damping I)
 * explicitly with the block layout of section 2.3 (block (j,j') of K is
 * At[j][j'] * Bt), solve K p = vec(G) with vec stacking the columns of the
 * d_out x d_in matrix G, and return p reshaped to d_out x d_in (row-major).
 * Returns the Cholesky status of K. */
int64_t oracle_kron_solve(const double *a, int64_t d_in, const double *b, int64_t d_out,
                          double damping, const double *grad, double *out)
{
    const int64_t n = d_in * d_out;
    double *k = (double *)malloc((size_t)n * n * sizeof(double));
    double *l = (double *)malloc((size_t)n * n * sizeof(double));
    double *v = (double *)malloc((size_t)n * sizeof(double));
    for (int64_t j = 0; j < d_in; ++j)
        for (int64_t i = 0; i < d_out; ++i)
            for (int64_t j2 = 0; j2 < d_in; ++j2)
                for (int64_t i2 = 0; i2 < d_out; ++i2) {
                    const double at = a[j * d_in + j2] + ((j == j2) ? damping : 0.0);
                    const double bt = b[i * d_out + i2] + ((i == i2) ? damping : 0.0);
                    k[(j * d_out + i) * n + (j2 * d_out + i2)] = at * bt;
                }
    for (int64_t j = 0; j < d_in; ++j)
        for (int64_t i = 0; i < d_out; ++i) v[j * d_out + i] = grad[i * d_in + j];
    const int64_t info = oracle_cholesky(k, n, n, l, n);
    if (info == 0) {
        for (int64_t i = 0; i < n; ++i) { /* l y = v */
            double s = v[i];
            for (int64_t c = 0; c < i; ++c) s -= l[i * n + c] * v[c];
            v[i] = s / l[i * n + i];
        }
        for (int64_t i = n - 1; i >= 0; --i) { /* l^T p = y */
            double s = v[i];
            for (int64_t c = i + 1; c < n; ++c) s -= l[c * n + i] * v[c];
            v[i] = s / l[i * n + i];
        }
        for (int64_t j = 0; j < d_in; ++j)
            for (int64_t i = 0; i < d_out; ++i) out[i * d_in + j] = v[j * d_out + i];
    }
    free(k);
    free(l);
    free(v);
    return info;
}
