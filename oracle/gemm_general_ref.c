/*
 * CPU oracle for the full row-major GEMM signature,
 *
 *     C  <-  alpha * op(A) * op(B) + beta * C,      op(X) = X or X^T,
 *
 * in binary64 (gemm_f64_general_ref) and binary32 (gemm_f32_general_ref).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT. Only the test-suite,
 * the smoke check and the benchmark's cpu-baseline leg may call it. It shares
 * no code, header, table or helper with the HIP library and never will.
 *
 * Where it comes from: the paper's Section 2.15 (Q4) states that DGEMM is
 * really C = alpha*A*B + beta*C, that its own study fixes alpha = beta = 1,
 * that the nests belonging to alpha or beta equal to 0 or 1 fold away, and
 * that strides and transposes are layout maps on the operands (Section 2.2:
 * a layout map turns the logical index pair into the stored one; (d0, d1) ->
 * (d1, d0) is the transpose).  The paper gives no arithmetic for alpha and
 * beta, so the definition is written out term by term, each operation rounded
 * once (round-to-nearest-even, no fused multiply-add; compile with
 * -ffp-contract=off and without fast-math):
 *
 *     s    = 0;  for k = 0 .. K-1 ascending:  p = opA(i,k) * opB(k,j);  s = s + p
 *     t    = alpha * s
 *     C_ij = t                          if beta == 0   (C is not read: it may hold anything)
 *     C_ij = t + beta * C_ij            otherwise      (product rounded, then the sum)
 *
 * and, as the folding remark implies, alpha == 0 (or K == 0) means that A and
 * B are not read at all:  C_ij = beta * C_ij  (+0 when beta == 0).
 *
 * Stored element of the operands (leading dimensions in elements):
 *     transa == 0:  A is M x K,  opA(i,k) = A[i*lda + k],  lda >= max(1, K)
 *     transa == 1:  A is K x M,  opA(i,k) = A[k*lda + i],  lda >= max(1, M)
 *     transb == 0:  B is K x N,  opB(k,j) = B[k*ldb + j],  ldb >= max(1, N)
 *     transb == 1:  B is N x K,  opB(k,j) = B[j*ldb + k],  ldb >= max(1, K)
 *     C is M x N,   C[i*ldc + j],                           ldc >= max(1, N)
 *
 * The loop order is i, k, j with one row of running sums s[0..N-1]; every
 * (i, j) still sees k ascending, and rows are independent (OpenMP over i), so
 * the result is that of the i, j, k nest bit for bit for any thread count.
 *
 * With alpha = beta = 1 and no transposes this is NOT the sequence of
 * gemm_f64_ref (which starts the sum from C): the two agree bit for bit only
 * when every partial sum is exact, and within rounding error otherwise.
 *
 * Pins (tests/test_oracle_general_pins.py): exact rational arithmetic on tiny
 * shapes for all four transpose combinations and dyadic alpha, beta; a
 * step-by-step correctly rounded emulation on random doubles; hand-derived
 * rounding cases; closed forms; NaN-filled operands that must not be read;
 * the recursive-summation error bound; planted mistakes.
 *
 * Return: 0 ok; -1 negative dimension or a trans flag other than 0/1; -2/-3/-4
 * lda/ldb/ldc too small; -5 null pointer for an operand that is read or
 * written; -10 out of memory for the row of running sums.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

static int check_general(int transa, int transb, int64_t M, int64_t N, int64_t K,
                         int a_read, const void *A, int64_t lda, const void *B,
                         int64_t ldb, const void *C, int64_t ldc)
{
    if (M < 0 || N < 0 || K < 0) return -1;
    if ((transa != 0 && transa != 1) || (transb != 0 && transb != 1)) return -1;
    const int64_t a_width = transa ? M : K, b_width = transb ? K : N;
    if (lda < (a_width > 1 ? a_width : 1)) return -2;
    if (ldb < (b_width > 1 ? b_width : 1)) return -3;
    if (ldc < (N > 1 ? N : 1)) return -4;
    if (M > 0 && N > 0 && C == NULL) return -5;
    if (M > 0 && N > 0 && K > 0 && a_read && (A == NULL || B == NULL)) return -5;
    return 0;
}

int gemm_f64_general_ref(int transa, int transb, int64_t M, int64_t N, int64_t K,
                         double alpha, const double *A, int64_t lda,
                         const double *B, int64_t ldb, double beta, double *C,
                         int64_t ldc)
{
    const int product = (alpha != 0.0) && K > 0;
    int rc = check_general(transa, transb, M, N, K, product, A, lda, B, ldb, C, ldc);
    if (rc) return rc;
    if (M == 0 || N == 0) return 0;
    if (!product) {
        for (int64_t i = 0; i < M; ++i)
            for (int64_t j = 0; j < N; ++j)
                C[i * ldc + j] = (beta == 0.0) ? 0.0 : beta * C[i * ldc + j];
        return 0;
    }
    int failed = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc((size_t)N * sizeof(double));
        if (!s) {
#pragma omp atomic write
            failed = 1;
        }
        int64_t i;
#pragma omp for schedule(static)
        for (i = 0; i < M; ++i) {
            if (!s) continue;
            for (int64_t j = 0; j < N; ++j) s[j] = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const double a = transa ? A[k * lda + i] : A[i * lda + k];
                for (int64_t j = 0; j < N; ++j) {
                    const double b = transb ? B[j * ldb + k] : B[k * ldb + j];
                    double p = a * b;
                    s[j] = s[j] + p;
                }
            }
            for (int64_t j = 0; j < N; ++j) {
                double t = alpha * s[j];
                if (beta == 0.0) {
                    C[i * ldc + j] = t;
                } else {
                    double u = beta * C[i * ldc + j];
                    C[i * ldc + j] = t + u;
                }
            }
        }
        free(s);
    }
    return failed ? -10 : 0;
}

int gemm_f32_general_ref(int transa, int transb, int64_t M, int64_t N, int64_t K,
                         float alpha, const float *A, int64_t lda, const float *B,
                         int64_t ldb, float beta, float *C, int64_t ldc)
{
    const int product = (alpha != 0.0f) && K > 0;
    int rc = check_general(transa, transb, M, N, K, product, A, lda, B, ldb, C, ldc);
    if (rc) return rc;
    if (M == 0 || N == 0) return 0;
    if (!product) {
        for (int64_t i = 0; i < M; ++i)
            for (int64_t j = 0; j < N; ++j)
                C[i * ldc + j] = (beta == 0.0f) ? 0.0f : beta * C[i * ldc + j];
        return 0;
    }
    int failed = 0;
#pragma omp parallel
    {
        float *s = (float *)malloc((size_t)N * sizeof(float));
        if (!s) {
#pragma omp atomic write
            failed = 1;
        }
        int64_t i;
#pragma omp for schedule(static)
        for (i = 0; i < M; ++i) {
            if (!s) continue;
            for (int64_t j = 0; j < N; ++j) s[j] = 0.0f;
            for (int64_t k = 0; k < K; ++k) {
                const float a = transa ? A[k * lda + i] : A[i * lda + k];
                for (int64_t j = 0; j < N; ++j) {
                    const float b = transb ? B[j * ldb + k] : B[k * ldb + j];
                    float p = a * b;
                    s[j] = s[j] + p;
                }
            }
            for (int64_t j = 0; j < N; ++j) {
                float t = alpha * s[j];
                if (beta == 0.0f) {
                    C[i * ldc + j] = t;
                } else {
                    float u = beta * C[i * ldc + j];
                    C[i * ldc + j] = t + u;
                }
            }
        }
        free(s);
    }
    return failed ? -10 : 0;
}
