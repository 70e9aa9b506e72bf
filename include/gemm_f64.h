/*
 * gemm_f64.h -- C ABI of libgemm_f64.so: double-precision GEMM for AMD MI355X (gfx950).
 *
 * The operation is the one the paper optimises (Section 2.1 "Affine Ops": the
 * canonical i, j, k nest  C[i][j] = C[i][j] + A[i][k] * B[k][j]  on three
 * row-major f64 buffers, C read and written in place; Section 2.2: the identity
 * layout map is row-major; Section 2.15 Q4: alpha = beta = 1 are assumed and
 * strides are the only layout generality kept):
 *
 *      C[i*ldc + j] += sum_{k=0}^{K-1} A[i*lda + k] * B[k*ldb + j],   0 <= i < M, 0 <= j < N.
 *
 * All matrix pointers are DEVICE pointers; leading dimensions count elements.
 * Every step of the computation runs in this library's own HIP kernels
 * (FP64 MFMA accumulator tiles, A/B panels staged through LDS, explicit edge
 * tiles); there is no host fallback and no dependency on a BLAS library.
 */
#ifndef GEMM_F64_H
#define GEMM_F64_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Return codes (0 = success; on any error nothing has been launched). */
enum {
    GEMM_F64_OK = 0,
    GEMM_F64_ERR_DIM = -1,       /* M, N or K negative, or a transpose flag other than 0/1 */
    GEMM_F64_ERR_LDA = -2,       /* lda < max(1, stored row length of A): K, or M if transposed */
    GEMM_F64_ERR_LDB = -3,       /* ldb < max(1, stored row length of B): N, or K if transposed */
    GEMM_F64_ERR_LDC = -4,       /* ldc < max(1, N)                                      */
    GEMM_F64_ERR_NULL = -5,      /* null pointer for an operand that has elements        */
    GEMM_F64_ERR_ALIGN = -6,     /* a pointer is not 8-byte aligned                      */
    GEMM_F64_ERR_LAUNCH = -7,    /* the HIP runtime refused the launch (see hipGetLastError) */
    GEMM_F64_ERR_TOO_LARGE = -8, /* M, N or K above 2^31 - 129 (32-bit tile arithmetic)     */
    GEMM_F64_ERR_VARIANT = -9,   /* unknown kernel variant index                         */
    GEMM_F64_ERR_SCRATCH = -10   /* gemm_f64_general_static: the split this problem wants needs more than the
                                    library's fixed scratch buffer, or that buffer could not be located */
};

/*
 * gemm_f64: enqueue C += A * B on `stream` and return at once (asynchronous).
 *
 *   M, N, K   logical sizes: A is M x K, B is K x N, C is M x N.  Zero is allowed:
 *             M == 0 or N == 0 does nothing; K == 0 leaves C unchanged.
 *   A, lda    device pointer, row-major, element (i,k) at A[i*lda + k]; lda >= max(1,K).
 *   B, ldb    device pointer, row-major, element (k,j) at B[k*ldb + j]; ldb >= max(1,N).
 *   C, ldc    device pointer, row-major, element (i,j) at C[i*ldc + j]; ldc >= max(1,N);
 *             read and written in place.
 *   stream    a hipStream_t passed as void*; NULL means the default stream.
 *
 * Layout and ownership: the caller owns all three buffers; the library keeps no
 * pointer, allocates nothing, uses no workspace and has no global state, so it
 * may be called from several host threads.  Inside a row's ld span, elements at
 * column index >= the logical width (K for A, N for B and C) are never read and
 * never written, and nothing past the last logical element of the last row is
 * touched.  C must not overlap A or B; A and B may alias each other.
 *
 * Alignment: pointers must be 8-byte aligned; nothing more is asked.  Operands
 * with odd leading dimensions or bases that are not 16-byte aligned run the
 * same kernel (its 16-byte global->LDS copies only need element alignment).
 * Leading dimensions of 2^22 or more elements switch to a slower variant of
 * the kernel that addresses memory with 64-bit pointers (same result).
 *
 * Arithmetic: binary64 throughout.  Products are accumulated from zero in the
 * matrix unit, four k at a time, and C is added once at the end, so the
 * rounding differs from the sequential nest: results are bit-identical to it
 * whenever every partial sum is exact (e.g. small-integer data) and within
 * 1e-13 * sum_k |a_ik * b_kj| elementwise otherwise.  The zero padding the
 * kernel uses for ragged K is applied to both operands, so a live Inf or NaN
 * never meets a padded zero.  The matrix unit returns sums of products that are
 * themselves below the normal range (operands around 2^-540) as signed zeros;
 * subnormal values of C are kept.  The one rounded addition per element that
 * updates C is performed by the kernel's lanes or, for large problems in
 * ordinary memory of the same GPU, by the memory system: the same bits either way (see
 * gemm_f64_set_epilogue_mode, the only process-wide state in the library, a
 * diagnostic that defaults to automatic).
 *
 * Errors: a negative code from the enum above; no exception, no errno.
 */
int gemm_f64(int64_t M, int64_t N, int64_t K,
             const double *A, int64_t lda,
             const double *B, int64_t ldb,
             double *C, int64_t ldc,
             void *stream);

/*
 * gemm_f64_ex: the same operation with the kernel variant chosen by the caller
 * (Section 2.10 of the paper tunes M_C, K_C, M_R, N_R by hand per problem; here
 * the analogous parameters are the workgroup macro-tile and the wave tile).
 * variant == -1 selects automatically, exactly as gemm_f64 does.  Variant
 * indices run from 0 to gemm_f64_variant_count() - 1.
 */
int gemm_f64_ex(int64_t M, int64_t N, int64_t K,
                const double *A, int64_t lda,
                const double *B, int64_t ldb,
                double *C, int64_t ldc,
                void *stream, int variant);

/*
 * gemm_f64_general: the full operation that the paper names but does not study
 * (Section 2.15 Q4: DGEMM is really C = alpha*A*B + beta*C, its own experiments
 * fix alpha = beta = 1, the cases alpha, beta in {0, 1} fold away, and strides
 * and transposes are layout maps on the operands -- Section 2.2, where
 * (d0, d1) -> (d1, d0) is the transpose):
 *
 *      C[i*ldc + j] <- alpha * sum_{k<K} opA(i,k) * opB(k,j) + beta * C[i*ldc + j]
 *
 *   transa    0: A is M x K, opA(i,k) = A[i*lda + k], lda >= max(1,K);
 *             1: A is stored transposed, K x M, opA(i,k) = A[k*lda + i], lda >= max(1,M).
 *   transb    0: B is K x N, opB(k,j) = B[k*ldb + j], ldb >= max(1,N);
 *             1: B is stored transposed, N x K, opB(k,j) = B[j*ldb + k], ldb >= max(1,K).
 *   alpha, beta   host scalars, passed by value.
 *   everything else as for gemm_f64 (device pointers, row-major, asynchronous on
 *   `stream`, no allocation, no workspace, padding inside a row's ld span and
 *   memory past the last logical element never touched).
 *
 * Folding: when alpha == 0 or K == 0, A and B are not read (they may be NULL)
 * and C <- beta * C (nothing is launched when beta == 1; C is set to +0 when
 * beta == 0).  When beta == 0, C is not read: it may hold anything, NaN
 * included, and is overwritten.
 *
 * Arithmetic: the sum over k is accumulated from zero in the matrix unit, then
 * t = alpha * sum and C = t + beta * C, each operation rounded on its own (no
 * fused multiply-add in this tail); C = t when beta == 0.  With alpha = beta =
 * 1 and no transposes this is gemm_f64 bit for bit.  Against the term-by-term
 * evaluation with k ascending the result is bit-identical whenever every
 * intermediate value is exact and within
 * 1e-13 * (|alpha| * sum_k |opA(i,k) * opB(k,j)| + |beta * C_in|) otherwise.
 *
 * Transposed operands change only how panels are brought into LDS; all four
 * combinations run the same MFMA kernel at the same speed class.
 */
int gemm_f64_general(int transa, int transb, int64_t M, int64_t N, int64_t K,
                     double alpha, const double *A, int64_t lda,
                     const double *B, int64_t ldb,
                     double beta, double *C, int64_t ldc,
                     void *stream);

/* gemm_f64_general with the kernel variant chosen by the caller (-1 = automatic), as gemm_f64_ex. */
int gemm_f64_general_ex(int transa, int transb, int64_t M, int64_t N, int64_t K,
                        double alpha, const double *A, int64_t lda,
                        const double *B, int64_t ldb,
                        double beta, double *C, int64_t ldc,
                        void *stream, int variant);

/*
 * gemm_f64_strided: C <- alpha * A * B + beta * C with every operand addressed through a row stride and a column
 * stride, in elements:
 *
 *     A(i,k) = A[i*rsa + k*csa]   (M x K),   B(k,j) = B[k*rsb + j*csb]   (K x N),   C(i,j) = C[i*rsc + j*csc]   (M x N).
 *
 * The paper describes an operand as an index space plus an affine layout map into its buffer and names a matrix
 * with access strides 128 and 2 inside a larger buffer as an example (Section 2.9); strides and transposes of the
 * GEMM operands are such maps (Section 2.15 Q4).  Two strides cover row-major (cs == 1), column-major or
 * transposed (rs == 1), and every regularly sampled sub-matrix of either; callers that hold column-major data
 * (Fortran BLAS conventions) pass rs = 1, cs = leading dimension for all three operands.
 *
 *   strides     all >= 1 (GEMM_F64_ERR_LDA / _LDB / _LDC names the operand otherwise); the stride of an extent of
 *               0 or 1 is never used.  A and B are only read, so their elements may share memory (a stride smaller
 *               than the extent it steps over is allowed).  The elements of C must be distinct and the library only
 *               accepts layouts where that is evident: rsc >= csc*(N-1)+1, or csc >= rsc*(M-1)+1, or M <= 1 or
 *               N <= 1; anything else is GEMM_F64_ERR_LDC.
 *   pointers    device, 8-byte aligned, address of element (0,0); elements that the strides do not reach are never
 *               read and never written.  Folding of alpha == 0, K == 0 and beta == 0, the arithmetic of the
 *               scalar tail, the other error codes and the tolerance are those of gemm_f64_general.
 *
 * Speed: when each operand has a unit stride and its other stride covers the extent (a leading dimension), the
 * call is gemm_f64_general on the same buffers (a column-major C is computed as the transposed problem
 * C^T = B^T A^T, which adds the same products in the same order) and runs on the MFMA kernels at full speed.  Any
 * other layout runs on the same kernel in a mode that gathers A and B element by element into its staging buffers
 * and scatters C (the MFMA loop is the same, the memory accesses are not coalesced; about two thirds of the full
 * speed for operands sampled with stride 2).  In every case nothing outside the layouts is read or written.
 * gemm_f64_strided_path tells which of the two a call takes.
 */
int gemm_f64_strided(int64_t M, int64_t N, int64_t K,
                     double alpha, const double *A, int64_t rsa, int64_t csa,
                     const double *B, int64_t rsb, int64_t csb,
                     double beta, double *C, int64_t rsc, int64_t csc,
                     void *stream);

/*
 * gemm_f64_strided_path: the pure host-side rule behind gemm_f64_strided and gemm_f32_strided (no device is touched;
 * the choice of kernels per layout is the tuning question of the paper's Section 2.15 Q5 applied to the layout maps
 * of Section 2.9).  Returns
 *   1  the call runs as a call of the transposed signature on the same buffers;
 *   2  it runs on the same MFMA kernel in its sampled mode, because some operand has no unit stride or no leading
 *      dimension that covers its rows;
 *  <0  the code gemm_f64_strided would return for these sizes and strides (outputs untouched).
 * The outputs describe the problem that runs.  *swapped = 0: first operand F = A (M x K), second S = B (K x N),
 * output O = C (M x N).  *swapped = 1: the transposed problem C^T = B^T A^T runs (C is column-major, or its row
 * stride is the smaller one): F = B^T (N x K), S = A^T (K x M), O = C^T (N x M).  F(x,k) sits at
 * F[x * *lda + k * *es_a] when *transa == 0 and at F[k * *lda + x * *es_a] when *transa == 1; S(k,x) at
 * S[k * *ldb + x * *es_b] when *transb == 0 and at S[x * *ldb + k * *es_b] when *transb == 1; O(r,c) at
 * O[r * *ldc + c * *es_c].  *es_a == *es_b == *es_c == 1 whenever 1 is returned.  Output pointers may be NULL.
 */
int gemm_f64_strided_path(int64_t M, int64_t N, int64_t K,
                          int64_t rsa, int64_t csa, int64_t rsb, int64_t csb, int64_t rsc, int64_t csc,
                          int *swapped, int *transa, int *transb, int64_t *lda, int64_t *ldb, int64_t *ldc,
                          int64_t *es_a, int64_t *es_b, int64_t *es_c);

/*
 * gemm_f64_general_ws: gemm_f64_general with a workspace on offer (the paper's Section 2.15 Q5 asks how tuning
 * choices are to be made per problem; splitting the k range is the one choice that needs memory).  For problems of
 * few output tiles and a long k range the library may cut the range into S slices, compute the S partial products
 * into S dense M x N slabs of the workspace with one launch, and add them up in ascending order in a second launch
 * (the result is a pure function of the arguments and of the workspace size on offer, never of scheduling).
 * Whether and how it splits is decided by gemm_f64_split_k_plan; a problem that is not split that way may instead have
 * only its last few tiles computed in slices (gemm_f64_tail_split_plan); with workspace == NULL, with too little of it
 * or when neither would pay, the call is gemm_f64_general exactly.
 *
 *   workspace        device pointer, 8-byte aligned, workspace_bytes long; owned by the caller, used only between
 *                    the two launches of this call on `stream`, contents undefined afterwards; calls that share a
 *                    workspace must be ordered (same stream, or synchronised).  May be NULL with workspace_bytes 0.
 *   workspace_bytes  what the library may use; gemm_f64_split_k_workspace_bytes says what it would like.
 *
 * The library still allocates nothing.  Arithmetic: each slice is accumulated from zero in the matrix unit, the
 * slabs are added in ascending slice order in binary64, then the scalar tail of gemm_f64_general; same tolerance.
 */
int gemm_f64_general_ws(int transa, int transb, int64_t M, int64_t N, int64_t K,
                        double alpha, const double *A, int64_t lda,
                        const double *B, int64_t ldb,
                        double beta, double *C, int64_t ldc,
                        void *workspace, int64_t workspace_bytes, void *stream);

/*
 * gemm_f64_general_static: gemm_f64_general_ws for callers that can neither allocate device memory nor hold a
 * workspace of their own: code under HIP graph capture, tight serving loops, harnesses that forbid allocation.
 * The workspace is a fixed buffer of GEMM_F64_STATIC_SCRATCH_BYTES inside the library's device image (one copy per
 * GPU, held from the moment the library is loaded on that GPU until the process ends).  The call allocates nothing
 * and frees nothing; it launches the same kernels as gemm_f64_general_ws.
 *
 * Which plan runs: the one gemm_f64_general_ws would run with a workspace of exactly
 * gemm_f64_split_k_workspace_bytes(transa, transb, M, N, K, compute units) bytes, i.e. the plan the rule prefers
 * when memory is no object; the results of the two calls are identical bit for bit.  If that plan needs more than
 * GEMM_F64_STATIC_SCRATCH_BYTES the call returns GEMM_F64_ERR_SCRATCH and launches nothing (use
 * gemm_f64_general_ws with a workspace of your own, or gemm_f64_general).  A problem the rule would not split
 * does not touch the buffer.  GEMM_F64_ERR_SCRATCH is also returned if the runtime cannot give the address of the
 * buffer on the current device (looked up once per device, on the first call there).
 *
 * The buffer keeps whatever the last call left in it; nothing in it needs to start from zero, because the first
 * launch of a split overwrites every element of every slab that the second launch reads.  Every call on a GPU
 * shares that GPU's buffer: calls that may overlap in time on one GPU (different streams without an ordering
 * between them, or host threads launching at once) race on it and must be ordered by the caller.
 * All other arguments, folding rules, error codes and the tolerance are those of gemm_f64_general_ws.
 */
#define GEMM_F64_STATIC_SCRATCH_BYTES (64ll << 20)
int gemm_f64_general_static(int transa, int transb, int64_t M, int64_t N, int64_t K,
                            double alpha, const double *A, int64_t lda,
                            const double *B, int64_t ldb,
                            double beta, double *C, int64_t ldc, void *stream);

/*
 * gemm_f64_split_k_plan: the pure host-side rule behind gemm_f64_general_ws (no device is touched).  Writes the
 * kernel variant, the number of slices (1 = the k range is not split) and the slice length (a multiple of 16;
 * K itself when not split) that a call with these arguments and this much workspace uses.  num_cu as for
 * gemm_f64_choose_variant.  Returns GEMM_F64_ERR_DIM for negative sizes or bad flags.
 */
int gemm_f64_split_k_plan(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu,
                          int64_t workspace_bytes, int *variant, int *splits, int *k_chunk);

/*
 * gemm_f64_tail_split_plan: the other use gemm_f64_general_ws makes of a workspace, again a pure host-side rule (the
 * partial-tile question of the paper's Section 2.15 Q2 at the level of the whole chip).  Workgroups run in rounds of
 * (compute units x resident workgroups); when the tiles of a problem make up whole rounds plus a small rest, that rest
 * would occupy a few compute units for the time of a whole tile.  Instead the last *tail_tiles tiles of the tile order
 * are computed in *tail_splits slices of the k range, *tail_k_chunk long each (a multiple of 16), into dense slabs of
 * the workspace, by extra workgroups of the same launch; a second, small launch adds the slabs of each tile in
 * ascending order and applies alpha and beta.  *tail_tiles == 0: no tail split (also whenever the k range of the whole
 * problem is split instead, see gemm_f64_split_k_plan; the two are never combined).  *variant is the kernel variant
 * of the call.  Arithmetic of the affected tiles: as for split K.  Returns GEMM_F64_ERR_DIM for negative sizes or
 * bad flags.  Output pointers may be NULL.
 */
int gemm_f64_tail_split_plan(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu,
                             int64_t workspace_bytes, int *variant, int *tail_tiles, int *tail_splits, int *tail_k_chunk);

/* Bytes of workspace the two rules together would use if they could have any amount (0: neither applies). */
int64_t gemm_f64_split_k_workspace_bytes(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu);

/*
 * Number of kernel variants and their names ("naive", "mfma_128x128x16", "mfma_64x64x16",
 * "mfma_128x64x16", "mfma_64x128x16", "mfma_32x64x16", "mfma_64x32x16"; NULL if out of range).
 * A 32-wide side needs the operand on that side to be contiguous along k: "mfma_32x64x16" exists for
 * transa == 0 only and "mfma_64x32x16" for transb == 1 only; asking for one with the other layout
 * returns GEMM_F64_ERR_VARIANT.
 */
int gemm_f64_variant_count(void);
const char *gemm_f64_variant_name(int variant);

/*
 * gemm_f64_choose_variant: the pure host-side selection rule used when
 * variant == -1 (the paper's Section 2.15 Q5 asks how parameters are to be
 * determined; this is a small analytical model: per variant, the larger of the tile-quantised makespan
 * at a measured efficiency and the time one tile needs on its own, which is what counts for problems
 * of fewer tiles than compute units).
 * num_cu is the number of compute units of the target device (256 on MI355X).
 * Touches no device.
 */
int gemm_f64_choose_variant(int64_t M, int64_t N, int64_t K, int num_cu);

/* The same rule for transposed operands (it only considers the variants that exist for the layout);
 * GEMM_F64_ERR_DIM if a flag is not 0 or 1. */
int gemm_f64_choose_variant_general(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu);

/*
 * gemm_f64_tile_of_block: the workgroup-id -> C-tile mapping used by the MFMA
 * kernels (the stand-in for the cache-level loop order of the paper's Section
 * 2.4 schedule).  Workgroups are handed to the 8 XCDs round-robin, so block b
 * runs on XCD b % 8; the mapping gives each XCD a contiguous run of a
 * grouped tile order so that tiles resident on one XCD share A and B panels
 * in that XCD's L2.  Pure host function; writes the tile coordinates of
 * `block` to *tile_m and *tile_n; returns 0, or GEMM_F64_ERR_DIM if the
 * arguments are out of range.
 */
int gemm_f64_tile_of_block(int64_t block, int64_t tiles_m, int64_t tiles_n,
                           int64_t *tile_m, int64_t *tile_n);

/*
 * gemm_f64_mfma_probe: a diagnostic, not part of the operation.  Enqueues a register-resident loop of
 * independent v_mfma_f64_16x16x4_f64 instructions with no memory traffic (two workgroups of four waves
 * per compute unit, sixteen accumulator tiles per wave, `iterations` rounds of sixteen instructions),
 * so that a benchmark can report what the matrix pipes sustain at the clock the chip actually holds
 * beside the published peak (the paper quotes its numbers against a machine peak in the same way,
 * Section 1.3).  `sink` is a device buffer of at least 512 * (compute units) elements that receives
 * one value per thread; *flops (host, may be NULL) receives the floating-point operations of the
 * launch.  Returns GEMM_F64_ERR_DIM for iterations outside 1 .. 2^30 or a sink that is too small.
 */
int gemm_f64_mfma_probe(int64_t iterations, double *sink, int64_t sink_elems, void *stream, double *flops);

/*
 * gemm_f64_device_peak: a diagnostic.  The matrix-pipe peaks of the current device computed as the paper computes
 * its machine peak (Section 1.2: arithmetic units x operations per cycle x clock): compute units x 4 SIMDs x 2048
 * flop per 16x16x4 MFMA / its issue cycles (64 in double, 32 in float) x the clock rate the device reports.  Any
 * output pointer (host) may be NULL.  256 units at 2.4 GHz give 78.6 and 157.3 TFLOP/s.  Returns
 * GEMM_F64_ERR_LAUNCH when the device cannot be queried.  Launches nothing.
 */
int gemm_f64_device_peak(int *compute_units, int *clock_khz, double *fp64_mfma_tflops, double *fp32_mfma_tflops);

/*
 * gemm_f64_set_epilogue_mode: a diagnostic switch for tests and measurements, process-wide, not meant for production
 * code (every other entry point is a pure function of its arguments).  With alpha == beta == 1 (the operation of the
 * paper's Section 2.1) the double-precision kernels update C in one of two ways that give the same bits: each lane
 * loads, adds and stores its elements, or it sends its sums to the memory system as floating-point additions without
 * return value (each element of C belongs to exactly one lane, so this is the same single rounding, and the order of
 * the additions is irrelevant).  The second form frees a workgroup's registers one memory latency earlier and is what
 * the library picks when K >= 256, C has at least 2^20 elements and C is ordinary device memory of the GPU the call
 * runs on.
 *   mode 0  automatic (the default);  1  always load, add, store;  2  additions in memory whenever C is such memory.
 * Returns the previous mode, or GEMM_F64_ERR_DIM for any other value.
 */
int gemm_f64_set_epilogue_mode(int mode);

/* Static description of a return code; never NULL, never freed. */
const char *gemm_f64_strerror(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int gemm_f64_version(void);

/*
 * A digest of the sources and compiler flags the library was built from (hexadecimal, static, never NULL; "unknown"
 * when the build did not provide one).  The build script compares it with the digest of the sources on disk to decide
 * whether a built library is out of date, independently of file times.
 */
const char *gemm_f64_build_id(void);

#ifdef __cplusplus
}
#endif
#endif /* GEMM_F64_H */
