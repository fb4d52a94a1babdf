/*
 * CPU oracle for single-precision general matrix multiply.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the definition written out: C = alpha * op(A) * op(B) + beta * C, where op(A) is M x K and
 * op(B) is K x N, which costs 2MNK floating-point operations (paper section 3.1, "SGEMM"; the interface is
 * that of Level-3 BLAS SGEMM, same section).  Three nested loops, the innermost a dot product taken in
 * index order p = 0..K-1.  No blocking, no packing, no vector code: it is meant to be checked by eye and it
 * plays the part of the "naive 3-loop matrix multiply" the paper times next to its kernel (section 3.4).
 *
 * Storage is ROW-major; a leading dimension is the distance in elements between consecutive rows (the
 * paper's "stride", section 3.4).  op(A)(i,p) = A[i*lda+p] for 'N' and A[p*lda+i] for 'T'.
 *
 * Two forms:
 *   ref_sgemm        float accumulator, float result, in place     -> the timed CPU baseline
 *   ref_sgemm_exact  double accumulator, double result, plus S_ij = sum_p |op(A)(i,p)| |op(B)(p,j)|
 *                    -> the reference value and the scale of the error bound
 * Only tests, the smoke check and the bench's cpu_baseline leg may use this file.  It shares nothing with
 * the HIP path.  The `omp parallel for` splits rows of C over host cores; it does not change any sum.
 */
#include <math.h>
#include <stddef.h>

static int is_n(char t) { return t == 'N' || t == 'n'; }
static int is_t(char t) { return t == 'T' || t == 't' || t == 'C' || t == 'c'; }

static int bad_args(char ta, char tb, int m, int n, int k, int lda, int ldb, int ldc)
{
    if (!(is_n(ta) || is_t(ta))) return 1;
    if (!(is_n(tb) || is_t(tb))) return 2;
    if (m < 0 || n < 0 || k < 0) return 3;
    int cols_a = is_n(ta) ? k : m;   /* row length of A as stored */
    int cols_b = is_n(tb) ? n : k;   /* row length of B as stored */
    if (lda < (cols_a > 1 ? cols_a : 1)) return 4;
    if (ldb < (cols_b > 1 ? cols_b : 1)) return 5;
    if (ldc < (n > 1 ? n : 1)) return 6;
    return 0;
}

int ref_sgemm(char ta, char tb, int m, int n, int k, float alpha, const float *A, int lda, const float *B,
              int ldb, float beta, float *C, int ldc)
{
    int bad = bad_args(ta, tb, m, n, k, lda, ldb, ldc);
    if (bad) return bad;
    const int an = is_n(ta), bn = is_n(tb);
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; ++i) {
        for (int j = 0; j < n; ++j) {
            float acc = 0.0f;
            for (int p = 0; p < k; ++p) {
                float a = an ? A[(size_t)i * lda + p] : A[(size_t)p * lda + i];
                float b = bn ? B[(size_t)p * ldb + j] : B[(size_t)j * ldb + p];
                acc += a * b;
            }
            float *c = &C[(size_t)i * ldc + j];
            /* beta == 0 means C is not read: whatever it held (NaN, Inf) must not reach the result */
            float old = (beta == 0.0f) ? 0.0f : beta * *c;
            *c = alpha * acc + old;
        }
    }
    return 0;
}

int ref_sgemm_exact(char ta, char tb, int m, int n, int k, float alpha, const float *A, int lda,
                    const float *B, int ldb, float beta, const float *C0, int ldc, double *Cref, double *S)
{
    int bad = bad_args(ta, tb, m, n, k, lda, ldb, ldc);
    if (bad) return bad;
    const int an = is_n(ta), bn = is_n(tb);
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; ++i) {
        for (int j = 0; j < n; ++j) {
            double acc = 0.0, mag = 0.0;
            for (int p = 0; p < k; ++p) {
                double a = an ? A[(size_t)i * lda + p] : A[(size_t)p * lda + i];
                double b = bn ? B[(size_t)p * ldb + j] : B[(size_t)j * ldb + p];
                acc += a * b;               /* a*b is exact in double for float a, b */
                mag += fabs(a) * fabs(b);
            }
            double old = (beta == 0.0f) ? 0.0 : (double)beta * (double)C0[(size_t)i * ldc + j];
            Cref[(size_t)i * n + j] = (double)alpha * acc + old;   /* Cref and S are dense m x n */
            if (S) S[(size_t)i * n + j] = mag;
        }
    }
    return 0;
}
