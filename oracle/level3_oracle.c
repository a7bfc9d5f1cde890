/*
 * CPU oracle for the GEMM-derived level-3 routines SYMM, SYRK and TRMM  --  TEST INFRASTRUCTURE,
 * NOT PRODUCT CODE.  Only tests, the smoke check and the benchmark's cpu_baseline leg may call this.
 * It shares no code, header, table or helper with the GPU library.
 *
 * The paper lists these routines in its routine table and says the gemm kernel family serves them
 * with the help of support kernels (Section 3.1); it gives no formulas, so the definitions are the
 * BLAS ones, written out as plain loops in FP64:
 *
 *   SYMM   C = alpha*A*B + beta*C  (side left,  A is m x m)   or
 *          C = alpha*B*A + beta*C  (side right, A is n x n);  C, B are m x n.
 *          A is symmetric and only its `uplo` triangle is read: A(i,j) with (i,j) outside that
 *          triangle is taken from the stored A(j,i).
 *   SYRK   C = alpha*A*A^T + beta*C  (trans none, A is n x k)   or
 *          C = alpha*A^T*A + beta*C  (trans,      A is k x n);  C is n x n and only its `uplo`
 *          triangle is read and written.  Entries outside it come back as NaN in c_ref (d_ref 0):
 *          the routine must leave them alone.
 *   TRMM   B = alpha*op(A)*B  (side left,  A is m x m)   or   B = alpha*B*op(A)  (side right,
 *          A is n x n);  B is m x n.  A is triangular: entries outside its `uplo` triangle count as
 *          zero and are not read; with a unit diagonal the stored diagonal is not read either and
 *          counts as one.
 *
 * Element (r,c) of a matrix with leading dimension ld lives at X[r + c*ld] (column-major) or
 * X[r*ld + c] (row-major).  beta == 0: C is not read; alpha == 0: A (and B for SYMM) are not read.
 * Outputs are dense FP64 arrays indexed [i*cols + j]; d_ref is the error denominator
 * |alpha| sum |a||b| + |beta||c_old| of the parity tests.  Sums run over the index l ascending.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#include "half_bits.h"

#define L3_ROW_MAJOR 101
#define L3_COL_MAJOR 102
#define L3_NO_TRANS 111
#define L3_UPPER 121
#define L3_LOWER 122
#define L3_NON_UNIT 131
#define L3_UNIT 132
#define L3_LEFT 141
#define L3_RIGHT 142

static double elem(int is_half, const void *base, size_t at)
{
    return is_half ? half_bits_to_double(((const uint16_t *)base)[at]) : (double)((const float *)base)[at];
}

static size_t where(int layout, int64_t r, int64_t c, int64_t ld)
{
    return layout == L3_COL_MAJOR ? (size_t)(r + c * ld) : (size_t)(r * ld + c);
}

static int inside(int uplo, int64_t r, int64_t c) { return uplo == L3_UPPER ? r <= c : r >= c; }

/* A(r,c) of a symmetric matrix of which only the uplo triangle is stored */
static double sym(int is_half, int layout, int uplo, const void *A, int64_t lda, int64_t r, int64_t c)
{
    return inside(uplo, r, c) ? elem(is_half, A, where(layout, r, c, lda)) : elem(is_half, A, where(layout, c, r, lda));
}

void oracle_symm(int is_half, int layout, int side, int uplo, int64_t m, int64_t n, double alpha, const void *A,
                 int64_t lda, const void *B, int64_t ldb, double beta, const void *C, int64_t ldc, double *c_ref,
                 double *d_ref)
{
    const int64_t inner = side == L3_LEFT ? m : n;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j) {
            double acc = 0.0, mag = 0.0;
            if (alpha != 0.0)
                for (int64_t l = 0; l < inner; ++l) {
                    double a, b;
                    if (side == L3_LEFT) {
                        a = sym(is_half, layout, uplo, A, lda, i, l);
                        b = elem(is_half, B, where(layout, l, j, ldb));
                    } else {
                        b = elem(is_half, B, where(layout, i, l, ldb));
                        a = sym(is_half, layout, uplo, A, lda, l, j);
                    }
                    acc += a * b;
                    mag += fabs(a) * fabs(b);
                }
            double r = alpha * acc, d = fabs(alpha) * mag;
            if (beta != 0.0) {
                const double o = elem(is_half, C, where(layout, i, j, ldc));
                r += beta * o;
                d += fabs(beta) * fabs(o);
            }
            c_ref[i * n + j] = r;
            d_ref[i * n + j] = d;
        }
}

void oracle_syrk(int is_half, int layout, int uplo, int trans, int64_t n, int64_t k, double alpha, const void *A,
                 int64_t lda, double beta, const void *C, int64_t ldc, double *c_ref, double *d_ref)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < n; ++j) {
            if (!inside(uplo, i, j)) {
                c_ref[i * n + j] = NAN;
                d_ref[i * n + j] = 0.0;
                continue;
            }
            double acc = 0.0, mag = 0.0;
            if (alpha != 0.0)
                for (int64_t l = 0; l < k; ++l) {
                    /* op(A) is n x k: row i times row j */
                    const double a = trans == L3_NO_TRANS ? elem(is_half, A, where(layout, i, l, lda))
                                                          : elem(is_half, A, where(layout, l, i, lda));
                    const double b = trans == L3_NO_TRANS ? elem(is_half, A, where(layout, j, l, lda))
                                                          : elem(is_half, A, where(layout, l, j, lda));
                    acc += a * b;
                    mag += fabs(a) * fabs(b);
                }
            double r = alpha * acc, d = fabs(alpha) * mag;
            if (beta != 0.0) {
                const double o = elem(is_half, C, where(layout, i, j, ldc));
                r += beta * o;
                d += fabs(beta) * fabs(o);
            }
            c_ref[i * n + j] = r;
            d_ref[i * n + j] = d;
        }
}

/* T(r,c) inside the triangle: one on a unit diagonal (the stored diagonal is then not read) */
static double tri(int is_half, int layout, int diag, const void *A, int64_t lda, int64_t r, int64_t c)
{
    if (r == c && diag == L3_UNIT) return 1.0;
    return elem(is_half, A, where(layout, r, c, lda));
}

void oracle_trmm(int is_half, int layout, int side, int uplo, int trans, int diag, int64_t m, int64_t n, double alpha,
                 const void *A, int64_t lda, const void *B, int64_t ldb, double *b_ref, double *d_ref)
{
    const int64_t inner = side == L3_LEFT ? m : n;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j) {
            double acc = 0.0, mag = 0.0;
            if (alpha != 0.0)
                for (int64_t l = 0; l < inner; ++l) {
                    /* left: op(A)(i,l) * B(l,j); right: B(i,l) * op(A)(l,j).  (r,c): where op(A)'s entry is stored */
                    int64_t r = side == L3_LEFT ? i : l, c = side == L3_LEFT ? l : j;
                    if (trans != L3_NO_TRANS) { const int64_t t = r; r = c; c = t; }
                    if (!inside(uplo, r, c)) continue;            /* a structural zero: no term */
                    const double a = tri(is_half, layout, diag, A, lda, r, c);
                    const double b = side == L3_LEFT ? elem(is_half, B, where(layout, l, j, ldb))
                                                     : elem(is_half, B, where(layout, i, l, ldb));
                    acc += a * b;
                    mag += fabs(a) * fabs(b);
                }
            b_ref[i * n + j] = alpha * acc;
            d_ref[i * n + j] = fabs(alpha) * mag;
        }
}
