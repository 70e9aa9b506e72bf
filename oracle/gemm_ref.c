/*
 * CPU oracle for double-precision GEMM, C += A*B, row-major.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT. Only the test-suite,
 * the smoke check and the benchmark's cpu-baseline leg may call it. It shares
 * no code, header, table or helper with the HIP library and never will.
 *
 * What it computes is the paper's canonical loop nest (Section 2.1, "Affine
 * Ops": three loops i, j, k around  c = c + a*b  written as a separate
 * multiply and add on f64 values of three row-major buffers, C read and
 * written in place; Section 2.15 Q4: alpha = beta = 1).  For every (i, j)
 *
 *     C[i*ldc + j]  <-  C[i*ldc + j] + sum_{k=0}^{K-1} A[i*lda + k] * B[k*ldb + j]
 *
 * evaluated in IEEE-754 binary64, round-to-nearest-even, with k ascending,
 * the product rounded first and the sum rounded second (two roundings, no
 * fused multiply-add; the translation unit must be compiled with
 * -ffp-contract=off and without any fast-math option).
 *
 * gemm_f64_ref      i-k-j loop order, OpenMP over rows.  Interchanging j and k
 *                   (Section 1.3 mentions ikj as the cache-friendly textbook
 *                   order) leaves the k-ascending sequence seen by each c_ij
 *                   untouched, and rows are independent, so the result is
 *                   bit-identical to the i-j-k nest for any thread count.
 * gemm_f64_ref_ijk  the nest exactly in the paper's loop order, serial; kept
 *                   so that a test can show the two agree bit for bit.
 * gemm_f64_absref   same loop on |a|, |b|: C += |A|*|B|.  With C = 0 on
 *                   entry it yields S_ij = sum_k |a_ik * b_kj|, the scale of
 *                   the elementwise tolerance used by the parity tests.
 *
 * Pins (tests/test_oracle_*.py): closed forms (all-ones operands, identity,
 * column sums, rank-1), exact rational arithmetic on tiny shapes, a
 * step-by-step correctly-rounded emulation, integer exactness against int64
 * matmul, the textbook recursive-summation error bound against exactly
 * rounded values, and k/row/column split invariants.
 *
 * Arguments are host pointers; leading dimensions are in elements.  Elements
 * with column index >= the logical width inside a row's ld span are neither
 * read nor written.  Return: 0 ok; -1 negative dimension; -2/-3/-4 lda/ldb/
 * ldc too small; -5 null pointer for a non-empty operand.
 */
#include <stddef.h>
#include <stdint.h>
#include <math.h>

#if defined(_OPENMP)
#include <omp.h>
#endif

static int check_args(int64_t M, int64_t N, int64_t K, const double *A,
                      int64_t lda, const double *B, int64_t ldb,
                      const double *C, int64_t ldc)
{
    if (M < 0 || N < 0 || K < 0) return -1;
    if (lda < (K > 1 ? K : 1)) return -2;
    if (ldb < (N > 1 ? N : 1)) return -3;
    if (ldc < (N > 1 ? N : 1)) return -4;
    if (M > 0 && N > 0 && C == NULL) return -5;
    if (M > 0 && N > 0 && K > 0 && (A == NULL || B == NULL)) return -5;
    return 0;
}

int gemm_f64_ref(int64_t M, int64_t N, int64_t K, const double *A, int64_t lda,
                 const double *B, int64_t ldb, double *C, int64_t ldc)
{
    int rc = check_args(M, N, K, A, lda, B, ldb, C, ldc);
    if (rc) return rc;
    if (M == 0 || N == 0 || K == 0) return 0;
    int64_t i;
#pragma omp parallel for schedule(static)
    for (i = 0; i < M; ++i) {
        double *c = C + i * ldc;
        for (int64_t k = 0; k < K; ++k) {
            const double a = A[i * lda + k];
            const double *b = B + k * ldb;
            for (int64_t j = 0; j < N; ++j) {
                double p = a * b[j];
                c[j] = c[j] + p;
            }
        }
    }
    return 0;
}

int gemm_f64_ref_ijk(int64_t M, int64_t N, int64_t K, const double *A,
                     int64_t lda, const double *B, int64_t ldb, double *C,
                     int64_t ldc)
{
    int rc = check_args(M, N, K, A, lda, B, ldb, C, ldc);
    if (rc) return rc;
    /* one running value per element: it starts from C, takes the K rounded products in ascending k, each
       addition rounded, and is stored once */
    for (int64_t i = 0; i < M; ++i) {
        const double *arow = A + i * lda;
        for (int64_t j = 0; j < N; ++j) {
            double acc = C[i * ldc + j];
            for (int64_t k = 0; k < K; ++k) {
                const double term = arow[k] * B[k * ldb + j];
                acc = acc + term;
            }
            C[i * ldc + j] = acc;
        }
    }
    return 0;
}

int gemm_f64_absref(int64_t M, int64_t N, int64_t K, const double *A,
                    int64_t lda, const double *B, int64_t ldb, double *C,
                    int64_t ldc)
{
    int rc = check_args(M, N, K, A, lda, B, ldb, C, ldc);
    if (rc) return rc;
    if (M == 0 || N == 0 || K == 0) return 0;
    int64_t i;
#pragma omp parallel for schedule(static)
    for (i = 0; i < M; ++i) {
        double *c = C + i * ldc;
        for (int64_t k = 0; k < K; ++k) {
            const double a = fabs(A[i * lda + k]);
            const double *b = B + k * ldb;
            for (int64_t j = 0; j < N; ++j) {
                double p = a * fabs(b[j]);
                c[j] = c[j] + p;
            }
        }
    }
    return 0;
}

/* Digest of the sources and flags this library was built from (set by oracle/build.py). */
#ifndef ORACLE_BUILD_ID
#define ORACLE_BUILD_ID "unknown"
#endif
const char *oracle_build_id(void)
{
    static const char tagged[] = "oracle-build-id:" ORACLE_BUILD_ID;
    return tagged + sizeof("oracle-build-id:") - 1;
}

/* Number of threads an OpenMP region of this library will use right now. */
int gemm_f64_ref_threads(void)
{
#if defined(_OPENMP)
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void gemm_f64_ref_set_threads(int n)
{
#if defined(_OPENMP)
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
