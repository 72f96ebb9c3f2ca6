/*
 * CPU oracle for the three dense kernels of the paper's case study (Section
 * "Linear Algebra Benchmarks"): 3mm  G = (A*B)*(C*D), LU decomposition without
 * pivoting  A = L*U, and Cholesky decomposition  A = L*L^T; and for solving
 * A*X = B with those factors by forward and backward substitution.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library is checked against.  It shares no code, header, table or helper with
 * the HIP path and nothing in the product path may call it.  Everything is
 * fp64, row-major (the paper's X[i, j] indexing in the 3mm tensor-expression
 * listing), leading dimensions in elements.
 *
 * Each routine is the textbook definition written as a plain loop nest: no
 * blocking, no fusion, no reordering of any sum.  Rows are independent inside
 * one elimination/column step, so the row loop carries an OpenMP pragma; the
 * order in which the terms of every single sum are added does not depend on
 * the thread count.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define IDX(i, j, ld) ((size_t)(i) * (size_t)(ld) + (size_t)(j))

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

/*
 * One matrix product  Out[i][j] = sum_{k=0..K-1} X[i][k] * Y[k][j], the sum
 * taken in ascending k (the paper's te.sum over the reduce axis, 3mm listing).
 * i-k-j loop order keeps the inner loop contiguous; for a fixed (i, j) the
 * terms are still added in ascending k.
 */
static void plain_product(const double *X, size_t ldx, const double *Y, size_t ldy,
                          double *Out, size_t ldo, int64_t rows, int64_t inner, int64_t cols)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        for (int64_t j = 0; j < cols; ++j) Out[IDX(i, j, ldo)] = 0.0;
        for (int64_t k = 0; k < inner; ++k) {
            const double x = X[IDX(i, k, ldx)];
            for (int64_t j = 0; j < cols; ++j)
                Out[IDX(i, j, ldo)] += x * Y[IDX(k, j, ldy)];
        }
    }
}

/*
 * 3mm (Section "Linear Algebra Benchmarks"; 3mm_basic listing):
 *   E = A*B   (ni x nj),  A ni x nk,  B nk x nj
 *   F = C*D   (nj x nl),  C nj x nm,  D nm x nl
 *   G = E*F   (ni x nl)
 * E and F are materialised fp64 arrays, exactly as in the listing, so they are
 * rounded to fp64 between the products.  All arrays dense (ld = columns).
 */
void oracle_mm3(const double *A, const double *B, const double *C, const double *D,
                double *E, double *F, double *G,
                int64_t ni, int64_t nk, int64_t nj, int64_t nm, int64_t nl)
{
    plain_product(A, (size_t)nk, B, (size_t)nj, E, (size_t)nj, ni, nk, nj);
    plain_product(C, (size_t)nm, D, (size_t)nl, F, (size_t)nl, nj, nm, nl);
    plain_product(E, (size_t)nj, F, (size_t)nl, G, (size_t)nl, ni, nj, nl);
}

/*
 * LU decomposition without pivoting, in place (Section "Linear Algebra
 * Benchmarks": A = L*U, L lower, U upper, no pivoting).  Reading taken where
 * the paper is silent: L has a unit diagonal that is not stored; on exit the
 * strict lower triangle holds L and the upper triangle with the diagonal
 * holds U.  Plain Gaussian elimination:
 *   for k: for i>k: a[i][k] /= a[k][k];  for i>k, j>k: a[i][j] -= a[i][k]*a[k][j]
 * Returns 0, or k+1 (1-based) for the first exactly-zero pivot, at which
 * point elimination stops and the remaining content is unspecified.
 */
int64_t oracle_lu(double *a, int64_t n, int64_t lda)
{
    for (int64_t k = 0; k < n; ++k) {
        const double pivot = a[IDX(k, k, lda)];
        if (pivot == 0.0) return k + 1;
#pragma omp parallel for schedule(static) if (n - k > 128)
        for (int64_t i = k + 1; i < n; ++i) {
            const double l = a[IDX(i, k, lda)] / pivot;
            a[IDX(i, k, lda)] = l;
            for (int64_t j = k + 1; j < n; ++j)
                a[IDX(i, j, lda)] -= l * a[IDX(k, j, lda)];
        }
    }
    return 0;
}

/*
 * Cholesky decomposition A = L*L^T (Section "Linear Algebra Benchmarks"), in
 * place, reading the lower triangle only.  Column by column:
 *   l[j][j] = sqrt(a[j][j] - sum_{k<j} l[j][k]^2)
 *   l[i][j] = (a[i][j] - sum_{k<j} l[i][k]*l[j][k]) / l[j][j]     (i > j)
 * Reading taken: on exit the lower triangle holds L and the strict upper
 * triangle is set to zero, so the output is literally the lower-triangular L.
 * Returns 0, or j+1 for the first pivot that is not strictly positive (NaN
 * included); content is then unspecified.
 */
int64_t oracle_cholesky(double *a, int64_t n, int64_t lda)
{
    for (int64_t j = 0; j < n; ++j) {
        double d = a[IDX(j, j, lda)];
        for (int64_t k = 0; k < j; ++k) d -= a[IDX(j, k, lda)] * a[IDX(j, k, lda)];
        if (!(d > 0.0)) return j + 1;
        const double ljj = sqrt(d);
        a[IDX(j, j, lda)] = ljj;
#pragma omp parallel for schedule(static) if (n - j > 128)
        for (int64_t i = j + 1; i < n; ++i) {
            double s = a[IDX(i, j, lda)];
            for (int64_t k = 0; k < j; ++k) s -= a[IDX(i, k, lda)] * a[IDX(j, k, lda)];
            a[IDX(i, j, lda)] = s / ljj;
        }
    }
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = i + 1; j < n; ++j) a[IDX(i, j, lda)] = 0.0;
    return 0;
}

/*
 * Backward residual of an in-place LU result:  ||A0 - L*U||_F / ||A0||_F with
 * L unit-lower from the strict lower triangle of lu and U from its upper
 * triangle.  (L*U)[i][j] = sum_{k<=min(i,j)} L[i][k]*U[k][j], written out.
 */
double oracle_lu_residual(const double *a0, int64_t lda0, const double *lu, int64_t ldlu, int64_t n)
{
    double num = 0.0, den = 0.0;
#pragma omp parallel for schedule(dynamic, 8) reduction(+ : num, den)
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t j = 0; j < n; ++j) {
            const int64_t kmax = i < j ? i : j;
            double s = 0.0;
            for (int64_t k = 0; k <= kmax; ++k) {
                const double l = (k == i) ? 1.0 : lu[IDX(i, k, ldlu)];
                s += l * lu[IDX(k, j, ldlu)];
            }
            const double r = a0[IDX(i, j, lda0)] - s;
            num += r * r;
            den += a0[IDX(i, j, lda0)] * a0[IDX(i, j, lda0)];
        }
    }
    return den > 0.0 ? sqrt(num / den) : sqrt(num);
}

/*
 * Backward residual of a Cholesky result:  ||A0 - L*L^T||_F / ||A0||_F, where
 * A0 is the symmetric matrix whose lower triangle was given (its upper
 * triangle is taken as the mirror image and never read) and L is the lower
 * triangle of l (its upper triangle is ignored here).
 */
double oracle_cholesky_residual(const double *a0, int64_t lda0, const double *l, int64_t ldl, int64_t n)
{
    double num = 0.0, den = 0.0;
#pragma omp parallel for schedule(dynamic, 8) reduction(+ : num, den)
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t j = 0; j <= i; ++j) {
            double s = 0.0;
            for (int64_t k = 0; k <= j; ++k) s += l[IDX(i, k, ldl)] * l[IDX(j, k, ldl)];
            const double aij = a0[IDX(i, j, lda0)];
            const double r = aij - s;
            const double w = (i == j) ? 1.0 : 2.0; /* mirrored entry counted too */
            num += w * r * r;
            den += w * aij * aij;
        }
    }
    return den > 0.0 ? sqrt(num / den) : sqrt(num);
}

/*
 * Matrix-vector forms used by the O(N^2) randomised reconstruction check at
 * sizes where the O(N^3) residual above is too slow:
 *   y = L*(U*x)   for an in-place LU result,
 *   y = L*(L^T*x) for a Cholesky result (lower triangle of l).
 * tmp is caller-provided scratch of n doubles.
 */
void oracle_lu_apply(const double *lu, int64_t ld, int64_t n, const double *x, double *tmp, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int64_t j = i; j < n; ++j) s += lu[IDX(i, j, ld)] * x[j];
        tmp[i] = s;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double s = tmp[i];
        for (int64_t j = 0; j < i; ++j) s += lu[IDX(i, j, ld)] * tmp[j];
        y[i] = s;
    }
}

void oracle_cholesky_apply(const double *l, int64_t ld, int64_t n, const double *x, double *tmp, double *y)
{
    for (int64_t j = 0; j < n; ++j) tmp[j] = 0.0;
    /* tmp = L^T x : tmp[j] = sum_{i>=j} l[i][j]*x[i]; row sweep keeps access contiguous */
    for (int64_t i = 0; i < n; ++i) {
        const double xi = x[i];
        for (int64_t j = 0; j <= i; ++j) tmp[j] += l[IDX(i, j, ld)] * xi;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int64_t j = 0; j <= i; ++j) s += l[IDX(i, j, ld)] * tmp[j];
        y[i] = s;
    }
}

/* y = A*x for a dense matrix, and y = S*x for the symmetric matrix given by its lower triangle. */
void oracle_matvec(const double *a, int64_t ld, int64_t rows, int64_t cols, const double *x, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        double s = 0.0;
        for (int64_t j = 0; j < cols; ++j) s += a[IDX(i, j, ld)] * x[j];
        y[i] = s;
    }
}

void oracle_symv_lower(const double *a, int64_t ld, int64_t n, const double *x, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int64_t j = 0; j <= i; ++j) s += a[IDX(i, j, ld)] * x[j];
        for (int64_t j = i + 1; j < n; ++j) s += a[IDX(j, i, ld)] * x[j];
        y[i] = s;
    }
}

/*
 * Solving A*X = B with the factors (the use the paper names for both
 * decompositions, Section "Introduction": solving systems of linear
 * equations).  B is n x nrhs, row-major, overwritten by X; every column is an
 * independent system, so the column loop carries the OpenMP pragma and each
 * column's sums are added in a fixed order.
 *
 *   LU:        L*y = b forward (unit diagonal: no division), then U*x = y backward.
 *   Cholesky:  L*y = b forward, then L^T*x = y backward (lower triangle of l only).
 */
void oracle_lu_solve(const double *lu, int64_t n, int64_t ld, double *b, int64_t nrhs, int64_t ldb)
{
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < nrhs; ++c) {
        for (int64_t i = 0; i < n; ++i) {
            double s = b[IDX(i, c, ldb)];
            for (int64_t j = 0; j < i; ++j) s -= lu[IDX(i, j, ld)] * b[IDX(j, c, ldb)];
            b[IDX(i, c, ldb)] = s;
        }
        for (int64_t i = n - 1; i >= 0; --i) {
            double s = b[IDX(i, c, ldb)];
            for (int64_t j = i + 1; j < n; ++j) s -= lu[IDX(i, j, ld)] * b[IDX(j, c, ldb)];
            b[IDX(i, c, ldb)] = s / lu[IDX(i, i, ld)];
        }
    }
}

void oracle_cholesky_solve(const double *l, int64_t n, int64_t ld, double *b, int64_t nrhs, int64_t ldb)
{
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < nrhs; ++c) {
        for (int64_t i = 0; i < n; ++i) {
            double s = b[IDX(i, c, ldb)];
            for (int64_t j = 0; j < i; ++j) s -= l[IDX(i, j, ld)] * b[IDX(j, c, ldb)];
            b[IDX(i, c, ldb)] = s / l[IDX(i, i, ld)];
        }
        for (int64_t i = n - 1; i >= 0; --i) {
            double s = b[IDX(i, c, ldb)];
            for (int64_t j = i + 1; j < n; ++j) s -= l[IDX(j, i, ld)] * b[IDX(j, c, ldb)];
            b[IDX(i, c, ldb)] = s / l[IDX(i, i, ld)];
        }
    }
}
