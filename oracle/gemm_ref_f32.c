/*
 * CPU oracle for single-precision GEMM, C += A*B, row-major.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT (same rules as gemm_ref.c: only the
 * test-suite, the smoke check and the benchmark's cpu-baseline leg may call it; no code is shared
 * with the HIP library).
 *
 * The paper obtains SGEMM from its DGEMM by substituting f32 for f64 in the operand types
 * (Section 2.13, "SGEMM performance"); the computation is therefore the loop nest of Section 2.1
 * with every value, product and sum in IEEE-754 binary32:
 *
 *     C[i*ldc + j]  <-  C[i*ldc + j] + sum_{k=0}^{K-1} A[i*lda + k] * B[k*ldb + j]
 *
 * k ascending, the product rounded to binary32 first and the sum rounded second (no fused
 * multiply-add, no wider intermediate: compile with -ffp-contract=off, no fast-math; on x86-64 the
 * float operations are SSE scalar/vector operations in binary32).
 *
 * gemm_f32_ref      i-k-j order, OpenMP over rows (bit-identical to the i-j-k nest, see gemm_ref.c).
 * gemm_f32_ref_ijk  the nest in the paper's loop order, serial.
 * gemm_f32_absref   S_ij += sum_k |a_ik * b_kj| accumulated in binary64 (S is a double matrix):
 *                   the scale of the elementwise tolerance; computed in double so that the scale
 *                   itself carries no visible error.
 *
 * Pins: the same families as for the double-precision oracle, re-derived for u = 2^-24
 * (tests/test_oracle_f32_pins.py).  Return codes as in gemm_ref.c.
 */
#include <stddef.h>
#include <stdint.h>
#include <math.h>

static int check_args32(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                        const void *C, int64_t ldc)
{
    if (M < 0 || N < 0 || K < 0) return -1;
    if (lda < (K > 1 ? K : 1)) return -2;
    if (ldb < (N > 1 ? N : 1)) return -3;
    if (ldc < (N > 1 ? N : 1)) return -4;
    if (M > 0 && N > 0 && C == NULL) return -5;
    if (M > 0 && N > 0 && K > 0 && (A == NULL || B == NULL)) return -5;
    return 0;
}

int gemm_f32_ref(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb, float *C,
                 int64_t ldc)
{
    int rc = check_args32(M, N, K, A, lda, B, ldb, C, ldc);
    if (rc) return rc;
    if (M == 0 || N == 0 || K == 0) return 0;
    int64_t i;
#pragma omp parallel for schedule(static)
    for (i = 0; i < M; ++i) {
        float *c = C + i * ldc;
        for (int64_t k = 0; k < K; ++k) {
            const float a = A[i * lda + k];
            const float *b = B + k * ldb;
            for (int64_t j = 0; j < N; ++j) {
                float p = a * b[j];
                c[j] = c[j] + p;
            }
        }
    }
    return 0;
}

int gemm_f32_ref_ijk(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb,
                     float *C, int64_t ldc)
{
    int rc = check_args32(M, N, K, A, lda, B, ldb, C, ldc);
    if (rc) return rc;
    for (int64_t i = 0; i < M; ++i) {
        const float *arow = A + i * lda;
        for (int64_t j = 0; j < N; ++j) {
            float acc = C[i * ldc + j];
            for (int64_t k = 0; k < K; ++k) {
                const float term = arow[k] * B[k * ldb + j];
                acc = acc + term;
            }
            C[i * ldc + j] = acc;
        }
    }
    return 0;
}

int gemm_f32_absref(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb,
                    double *S, int64_t lds)
{
    int rc = check_args32(M, N, K, A, lda, B, ldb, S, lds);
    if (rc) return rc;
    if (M == 0 || N == 0 || K == 0) return 0;
    int64_t i;
#pragma omp parallel for schedule(static)
    for (i = 0; i < M; ++i) {
        double *s = S + i * lds;
        for (int64_t k = 0; k < K; ++k) {
            const double a = fabs((double)A[i * lda + k]);
            const float *b = B + k * ldb;
            for (int64_t j = 0; j < N; ++j) s[j] = s[j] + a * fabs((double)b[j]);
        }
    }
    return 0;
}
