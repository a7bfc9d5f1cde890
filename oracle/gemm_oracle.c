/*
 * CPU oracle for GEMM and batched GEMM  --  TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this.
 * It shares no code, header, table or helper with the GPU library.
 *
 * What it computes is the textbook definition the paper relies on when it names
 * "GEMM" and "the BLAS API" (Section 1; Section 3.1 "Library Design"), written out
 * as a plain triple loop in FP64:
 *
 *     acc(i,j)  = sum_{l=0}^{k-1} opA(i,l) * opB(l,j)            (l ascending, FP64)
 *     C(i,j)    = alpha*acc(i,j) + beta*C_old(i,j)                (FP64)
 *     D(i,j)    = |alpha| * sum_l |opA(i,l)|*|opB(l,j)| + |beta|*|C_old(i,j)|
 *
 * opX = X or X^T.  A matrix element (r,c) with leading dimension ld lives at
 * X[r + c*ld] (column-major) or X[r*ld + c] (row-major); both layouts are indexed
 * directly, no operand swapping.  beta == 0 means C_old is not read at all;
 * alpha == 0 (or k == 0) means A and B are not read at all (BLAS convention).
 *
 * The batched form (Section 4.6 "Batched BLAS Routines") repeats the same thing per
 * instance with per-instance element offsets into A, B, C and per-instance alpha, beta.
 *
 * The matrix-vector product (Section 4.2 benchmarks it beside GEMM) is the same sum with a
 * single output column and strided vectors; it has a loop of its own, oracle_gemv.
 *
 * Outputs are dense FP64 arrays indexed [i*n + j] (and [b*m*n + i*n + j] when batched);
 * nothing is rounded to the storage type.  D is the denominator of the relative error
 * the parity tests use.
 *
 * Parallelism: OpenMP over output elements only; the inner loop is untouched.
 */
#include <stddef.h>
#include <stdint.h>
#include <math.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORA_ROW_MAJOR 101
#define ORA_COL_MAJOR 102
#define ORA_NO_TRANS 111
#define ORA_TRANS 112

#include "half_bits.h"

static inline double load_f32(const void *base, size_t at) { return (double)((const float *)base)[at]; }
static inline double load_f16(const void *base, size_t at) { return half_bits_to_double(((const uint16_t *)base)[at]); }

/* position of stored element (r,c) */
static inline size_t at(int layout, int64_t r, int64_t c, int64_t ld)
{
    return layout == ORA_COL_MAJOR ? (size_t)(r + c * ld) : (size_t)(r * ld + c);
}

/* one output element of the definition above */
static void one_entry(int is_half, int layout, int ta, int tb, int64_t k,
                      double alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                      double beta, const void *C, int64_t ldc,
                      int64_t i, int64_t j, double *c_out, double *d_out)
{
    double acc = 0.0, mag = 0.0;
    if (alpha != 0.0) {
        for (int64_t l = 0; l < k; ++l) {
            size_t pa = (ta == ORA_NO_TRANS) ? at(layout, i, l, lda) : at(layout, l, i, lda);
            size_t pb = (tb == ORA_NO_TRANS) ? at(layout, l, j, ldb) : at(layout, j, l, ldb);
            double a = is_half ? load_f16(A, pa) : load_f32(A, pa);
            double b = is_half ? load_f16(B, pb) : load_f32(B, pb);
            acc += a * b;
            mag += fabs(a) * fabs(b);
        }
    }
    double val = alpha * acc;
    double den = fabs(alpha) * mag;
    if (beta != 0.0) {
        size_t pc = at(layout, i, j, ldc);
        double c = is_half ? load_f16(C, pc) : load_f32(C, pc);
        val += beta * c;
        den += fabs(beta) * fabs(c);
    }
    *c_out = val;
    *d_out = den;
}

static void gemm_full(int is_half, int layout, int ta, int tb, int64_t m, int64_t n, int64_t k,
                      double alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                      double beta, const void *C, int64_t ldc, double *c_ref, double *d_ref)
{
    int64_t total = m * n;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < total; ++p) {
        int64_t i = p / n, j = p % n;
        one_entry(is_half, layout, ta, tb, k, alpha, A, lda, B, ldb, beta, C, ldc, i, j,
                  &c_ref[p], &d_ref[p]);
    }
}

/* ---- exported entry points (host pointers everywhere) ------------------------------- */

/* FP32 storage.  c_ref, d_ref: m*n doubles each, [i*n + j]. */
void oracle_sgemm(int layout, int ta, int tb, int64_t m, int64_t n, int64_t k,
                  double alpha, const float *A, int64_t lda, const float *B, int64_t ldb,
                  double beta, const float *C, int64_t ldc, double *c_ref, double *d_ref)
{
    gemm_full(0, layout, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, c_ref, d_ref);
}

/* FP16 storage given as raw binary16 bit patterns; values are widened exactly. */
void oracle_hgemm(int layout, int ta, int tb, int64_t m, int64_t n, int64_t k,
                  double alpha, const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
                  double beta, const uint16_t *C, int64_t ldc, double *c_ref, double *d_ref)
{
    gemm_full(1, layout, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, c_ref, d_ref);
}

/* Selected output entries only: sample s is element (rows[s], cols[s]).
 * Used where the full m*n*k loop is too slow; each entry is still the full-length sum. */
void oracle_gemm_entries(int is_half, int layout, int ta, int tb, int64_t k,
                         double alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                         double beta, const void *C, int64_t ldc,
                         const int64_t *rows, const int64_t *cols, int64_t count,
                         double *c_ref, double *d_ref)
{
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < count; ++s) {
        one_entry(is_half, layout, ta, tb, k, alpha, A, lda, B, ldb, beta, C, ldc,
                  rows[s], cols[s], &c_ref[s], &d_ref[s]);
    }
}

/* Batched FP32: instance b uses A + a_off[b], B + b_off[b], C + c_off[b] (element offsets),
 * alphas[b], betas[b]; all instances share layout, ops, m, n, k and leading dimensions.
 * c_ref, d_ref: batch*m*n doubles, [b*m*n + i*n + j]. */
void oracle_sgemm_batched(int layout, int ta, int tb, int64_t m, int64_t n, int64_t k,
                          const float *alphas, const float *A, const int64_t *a_off, int64_t lda,
                          const float *B, const int64_t *b_off, int64_t ldb,
                          const float *betas, const float *C, const int64_t *c_off, int64_t ldc,
                          int64_t batch, double *c_ref, double *d_ref)
{
    int64_t per = m * n;
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < batch * per; ++q) {
        int64_t b = q / per, p = q % per;
        int64_t i = p / n, j = p % n;
        one_entry(0, layout, ta, tb, k, (double)alphas[b], A + a_off[b], lda, B + b_off[b], ldb,
                  (double)betas[b], C + c_off[b], ldc, i, j, &c_ref[q], &d_ref[q]);
    }
}

/* Batched FP16 storage: the same per instance; A, B, C hold binary16 bit patterns, offsets are in
 * elements, alphas and betas are FP32 (the scalar type of the FP16 routines). */
void oracle_hgemm_batched(int layout, int ta, int tb, int64_t m, int64_t n, int64_t k,
                          const float *alphas, const uint16_t *A, const int64_t *a_off, int64_t lda,
                          const uint16_t *B, const int64_t *b_off, int64_t ldb,
                          const float *betas, const uint16_t *C, const int64_t *c_off, int64_t ldc,
                          int64_t batch, double *c_ref, double *d_ref)
{
    int64_t per = m * n;
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < batch * per; ++q) {
        int64_t b = q / per, p = q % per;
        int64_t i = p / n, j = p % n;
        one_entry(1, layout, ta, tb, k, (double)alphas[b], A + a_off[b], lda, B + b_off[b], ldb,
                  (double)betas[b], C + c_off[b], ldc, i, j, &c_ref[q], &d_ref[q]);
    }
}

/* Matrix-vector product (the level-2 routine the paper benchmarks next to GEMM, Section 4.2), BLAS GEMV:
 *     y(i) = alpha * sum_l op(A)(i,l) * x(l) + beta * y(i),     op(A) is M x K with (M, K) = (m, n) or (n, m)
 * A is m x n in the given layout with leading dimension lda; x(l) lives at x[l*incx], y(i) at y[i*incy]
 * (positive increments).  beta == 0: y is not read; alpha == 0: A and x are not read.
 * y_ref, d_ref: M doubles; d = |alpha| sum |op(A)(i,l)||x(l)| + |beta||y(i)|. */
void oracle_gemv(int is_half, int layout, int trans, int64_t m, int64_t n, double alpha, const void *A, int64_t lda,
                 const void *x, int64_t incx, double beta, const void *y, int64_t incy, double *y_ref, double *d_ref)
{
    const int64_t rows = trans == ORA_NO_TRANS ? m : n, len = trans == ORA_NO_TRANS ? n : m;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        double acc = 0.0, mag = 0.0;
        if (alpha != 0.0)
            for (int64_t l = 0; l < len; ++l) {
                const size_t pa = trans == ORA_NO_TRANS ? at(layout, i, l, lda) : at(layout, l, i, lda);
                const double a = is_half ? load_f16(A, pa) : load_f32(A, pa);
                const double v = is_half ? load_f16(x, (size_t)(l * incx)) : load_f32(x, (size_t)(l * incx));
                acc += a * v;
                mag += fabs(a) * fabs(v);
            }
        double r = alpha * acc, d = fabs(alpha) * mag;
        if (beta != 0.0) {
            const double o = is_half ? load_f16(y, (size_t)(i * incy)) : load_f32(y, (size_t)(i * incy));
            r += beta * o;
            d += fabs(beta) * fabs(o);
        }
        y_ref[i] = r;
        d_ref[i] = d;
    }
}

/* binary16 -> double for arrays (lets tests pin the converter on all 65536 patterns) */
void oracle_half_to_double(const uint16_t *src, int64_t count, double *dst)
{
    for (int64_t t = 0; t < count; ++t) dst[t] = half_bits_to_double(src[t]);
}

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
