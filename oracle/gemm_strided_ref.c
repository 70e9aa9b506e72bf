/*
 * CPU oracle for GEMM on operands addressed through two strides each,
 *
 *     C  <-  alpha * A * B + beta * C,
 *     A(i,k) = A[i*rsa + k*csa],  B(k,j) = B[k*rsb + j*csb],  C(i,j) = C[i*rsc + j*csc],
 *
 * in binary64 (gemm_f64_strided_ref) and binary32 (gemm_f32_strided_ref).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT. Only the test-suite,
 * the smoke check and the benchmark's cpu-baseline leg may call it. It shares
 * no code, header, table or helper with the HIP library and never will.
 *
 * Where it comes from: the paper's Section 2.9 describes an operand as a
 * logical index space plus an affine layout map into a buffer and gives the
 * map (d0, d1) -> (d0 * 128 + d1 * 2), a matrix with access strides 128 and 2
 * inside a larger buffer, as an example; Section 2.15 (Q4) says that strides
 * and transposes of the GEMM operands are exactly such maps.  A pair of
 * strides per operand covers row-major (cs = 1), column-major or transposed
 * (rs = 1) and every regularly sampled sub-matrix of either.  The arithmetic
 * is that of the full signature, written out term by term with every
 * operation rounded once (round-to-nearest-even, no fused multiply-add;
 * compile with -ffp-contract=off and without fast-math):
 *
 *     s    = 0;  for k = 0 .. K-1 ascending:  p = A(i,k) * B(k,j);  s = s + p
 *     t    = alpha * s
 *     C_ij = t                    if beta == 0   (C is not read)
 *     C_ij = t + beta * C_ij      otherwise
 *     alpha == 0 or K == 0:  A and B are not read,  C_ij = beta * C_ij  (+0 when beta == 0)
 *
 * Strides are in elements and at least 1.  The elements of C must be distinct:
 * accepted are layouts in which one stride spans the other's whole extent
 * (rsc >= csc*(N-1)+1, or csc >= rsc*(M-1)+1), and single rows or columns.
 * A and B are only read, so their elements may overlap in memory.
 *
 * Loop order i, k, j with one row of running sums; every (i, j) sees k
 * ascending and rows are independent (OpenMP over i), so the result is that
 * of the i, j, k nest bit for bit for any thread count.
 *
 * Pins (tests/test_oracle_strided_pins.py): exact rational arithmetic on tiny
 * shapes over row-major, column-major and sampled layouts of every operand;
 * every pin of the transposed signature re-expressed through strides, with C
 * row-major and column-major; exact integer products of sampled sub-matrices;
 * the paper's own example layout; operands that must not be read; planted
 * mistakes.
 *
 * Return: 0 ok; -1 negative dimension; -2/-3/-4 a stride of A/B/C below 1, or
 * a layout of C whose elements are not known to be distinct; -5 null pointer
 * for an operand that is read or written; -10 out of memory.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

static int check_strided(int64_t M, int64_t N, int64_t K, int ab_read, const void *A,
                         int64_t rsa, int64_t csa, const void *B, int64_t rsb,
                         int64_t csb, const void *C, int64_t rsc, int64_t csc)
{
    if (M < 0 || N < 0 || K < 0) return -1;
    if (rsa < 1 || csa < 1) return -2;
    if (rsb < 1 || csb < 1) return -3;
    if (rsc < 1 || csc < 1) return -4;
    if (M > 1 && N > 1) {
        /* in 128-bit arithmetic: the extents times the strides may exceed 64 bits */
        const __int128 row_span = (__int128)csc * (N - 1) + 1, col_span = (__int128)rsc * (M - 1) + 1;
        if (!((__int128)rsc >= row_span || (__int128)csc >= col_span)) return -4;
    }
    if (M > 0 && N > 0 && C == NULL) return -5;
    if (M > 0 && N > 0 && K > 0 && ab_read && (A == NULL || B == NULL)) return -5;
    return 0;
}

int gemm_f64_strided_ref(int64_t M, int64_t N, int64_t K, double alpha, const double *A,
                         int64_t rsa, int64_t csa, const double *B, int64_t rsb,
                         int64_t csb, double beta, double *C, int64_t rsc, int64_t csc)
{
    const int product = (alpha != 0.0) && K > 0;
    int rc = check_strided(M, N, K, product, A, rsa, csa, B, rsb, csb, C, rsc, csc);
    if (rc) return rc;
    if (M == 0 || N == 0) return 0;
    if (!product) {
        for (int64_t i = 0; i < M; ++i)
            for (int64_t j = 0; j < N; ++j) {
                double *c = C + i * rsc + j * csc;
                *c = (beta == 0.0) ? 0.0 : beta * *c;
            }
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
                const double a = A[i * rsa + k * csa];
                for (int64_t j = 0; j < N; ++j) {
                    double p = a * B[k * rsb + j * csb];
                    s[j] = s[j] + p;
                }
            }
            for (int64_t j = 0; j < N; ++j) {
                double *c = C + i * rsc + j * csc;
                double t = alpha * s[j];
                if (beta == 0.0) {
                    *c = t;
                } else {
                    double u = beta * *c;
                    *c = t + u;
                }
            }
        }
        free(s);
    }
    return failed ? -10 : 0;
}

int gemm_f32_strided_ref(int64_t M, int64_t N, int64_t K, float alpha, const float *A,
                         int64_t rsa, int64_t csa, const float *B, int64_t rsb,
                         int64_t csb, float beta, float *C, int64_t rsc, int64_t csc)
{
    const int product = (alpha != 0.0f) && K > 0;
    int rc = check_strided(M, N, K, product, A, rsa, csa, B, rsb, csb, C, rsc, csc);
    if (rc) return rc;
    if (M == 0 || N == 0) return 0;
    if (!product) {
        for (int64_t i = 0; i < M; ++i)
            for (int64_t j = 0; j < N; ++j) {
                float *c = C + i * rsc + j * csc;
                *c = (beta == 0.0f) ? 0.0f : beta * *c;
            }
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
                const float a = A[i * rsa + k * csa];
                for (int64_t j = 0; j < N; ++j) {
                    float p = a * B[k * rsb + j * csb];
                    s[j] = s[j] + p;
                }
            }
            for (int64_t j = 0; j < N; ++j) {
                float *c = C + i * rsc + j * csc;
                float t = alpha * s[j];
                if (beta == 0.0f) {
                    *c = t;
                } else {
                    float u = beta * *c;
                    *c = t + u;
                }
            }
        }
        free(s);
    }
    return failed ? -10 : 0;
}
