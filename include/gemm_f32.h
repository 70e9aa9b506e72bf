/*
 * gemm_f32.h -- single-precision entry points of libgemm_f64.so (AMD MI355X, gfx950).
 *
 * The paper derives SGEMM from its DGEMM by substituting f32 for f64 in the operand types and
 * doubling the elements per vector register (Section 2.13, "SGEMM performance"); the operation is
 * the loop nest of Section 2.1 on float buffers:
 *
 *      C[i*ldc + j] += sum_{k=0}^{K-1} A[i*lda + k] * B[k*ldb + j],   0 <= i < M, 0 <= j < N.
 *
 * Everything stated in gemm_f64.h about argument meaning, layout, ownership, asynchrony, aliasing,
 * edge handling and error behaviour holds here with `float` for `double`; the return codes are the
 * GEMM_F64_* values of that header.  Differences:
 *   - pointers must be 4-byte aligned, nothing more; leading dimensions of 2^23 or more elements
 *     switch to the slower 64-bit-addressing variant of the kernel (same result);
 *   - arithmetic is binary32 throughout (FP32 MFMA, four k per instruction, accumulated from zero,
 *     C added once at the end): bit-identical to the sequential binary32 nest whenever every
 *     partial sum is exact (e.g. integer data with |sum| < 2^24), and within
 *     2^-19 * sum_k |a_ik * b_kj| of it elementwise otherwise (both are within the recursive
 *     summation bound of the exact result; the typical difference is about 2^-24 of that scale).
 */
#ifndef GEMM_F32_H
#define GEMM_F32_H

#include <stdint.h>

#include "gemm_f64.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Enqueue C += A * B (float, device pointers, row-major, leading dimensions in elements) on `stream`. */
int gemm_f32(int64_t M, int64_t N, int64_t K,
             const float *A, int64_t lda,
             const float *B, int64_t ldb,
             float *C, int64_t ldc,
             void *stream);

/* The same with an explicit kernel variant (-1 = automatic), as gemm_f64_ex. */
int gemm_f32_ex(int64_t M, int64_t N, int64_t K,
                const float *A, int64_t lda,
                const float *B, int64_t ldb,
                float *C, int64_t ldc,
                void *stream, int variant);

/*
 * The full operation C <- alpha * op(A) * op(B) + beta * C in float (Section 2.15 Q4 and Section 2.2 of
 * the paper, see gemm_f64_general for the argument meaning, the folding rules for alpha == 0, K == 0 and
 * beta == 0, and the arithmetic of the scalar tail).  Tolerance against the term-by-term binary32
 * evaluation: 2^-19 * (|alpha| * sum_k |opA(i,k) * opB(k,j)| + |beta * C_in|); bit-identical when every
 * intermediate value is exact.
 */
int gemm_f32_general(int transa, int transb, int64_t M, int64_t N, int64_t K,
                     float alpha, const float *A, int64_t lda,
                     const float *B, int64_t ldb,
                     float beta, float *C, int64_t ldc,
                     void *stream);
int gemm_f32_general_ex(int transa, int transb, int64_t M, int64_t N, int64_t K,
                        float alpha, const float *A, int64_t lda,
                        const float *B, int64_t ldb,
                        float beta, float *C, int64_t ldc,
                        void *stream, int variant);

/* The float counterpart of gemm_f64_strided (operands addressed through a row and a column stride each, Section 2.9
 * and Section 2.15 Q4 of the paper; pointers 4-byte aligned; tolerance of gemm_f32_general). */
int gemm_f32_strided(int64_t M, int64_t N, int64_t K,
                     float alpha, const float *A, int64_t rsa, int64_t csa,
                     const float *B, int64_t rsb, int64_t csb,
                     float beta, float *C, int64_t rsc, int64_t csc,
                     void *stream);

/* The float counterparts of gemm_f64_general_ws, gemm_f64_split_k_plan, gemm_f64_tail_split_plan and
 * gemm_f64_split_k_workspace_bytes (workspace 4-byte aligned, slice lengths multiples of 32). */
int gemm_f32_general_ws(int transa, int transb, int64_t M, int64_t N, int64_t K,
                        float alpha, const float *A, int64_t lda,
                        const float *B, int64_t ldb,
                        float beta, float *C, int64_t ldc,
                        void *workspace, int64_t workspace_bytes, void *stream);
int gemm_f32_split_k_plan(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu,
                          int64_t workspace_bytes, int *variant, int *splits, int *k_chunk);
int gemm_f32_tail_split_plan(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu,
                             int64_t workspace_bytes, int *variant, int *tail_tiles, int *tail_splits, int *tail_k_chunk);
int64_t gemm_f32_split_k_workspace_bytes(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu);

/* Variant table of the float kernels ("mfma_128x128x32", ...) and the host-side selection rule
 * (the analogue of choosing M_C, K_C, M_R, N_R per element type in Section 2.13). */
int gemm_f32_variant_count(void);
const char *gemm_f32_variant_name(int variant);
int gemm_f32_choose_variant(int64_t M, int64_t N, int64_t K, int num_cu);
int gemm_f32_choose_variant_general(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu);

/* The float counterpart of gemm_f64_mfma_probe (v_mfma_f32_16x16x4_f32). */
int gemm_f32_mfma_probe(int64_t iterations, float *sink, int64_t sink_elems, void *stream, double *flops);

#ifdef __cplusplus
}
#endif
#endif /* GEMM_F32_H */
