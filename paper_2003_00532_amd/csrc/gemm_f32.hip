// libgemm_f64.so, single-precision entry points (declared and documented in include/gemm_f32.h).
#include "../../include/gemm_f32.h"

#include "gemm_host.hpp"

using namespace gemm_detail;

namespace {
// Index order is part of the ABI of gemm_f32_ex.  One LDS stage holds 32 values of k in float.
// The parameters of the selection model are the ones fitted for the double kernels: in units of MFMA issue slots the
// two precisions behave alike (at 8192^3 the float kernels reach 95.2 / 93.4 / 94.5 / 95.7 % of the FP32 peak with the
// 128x128 / 64x64 / 128x64 / 64x128 tiles).  What was measured in float is the outcome: over the 17 shapes of
// `bench.py --selection-study --dtype f32` the variant chosen with these parameters is 1.2 % slower than the best
// variant on average on one machine of the pool and 1.6 % on another (largest: 2304^3, 9.7 to 13.4 %).
const Variant kVariants[] = {
    {"naive", 0, 0, 0.0, 1, 0.0},
    {"mfma_128x128x32", 128, 128, 0.955, 2, 286.0},
    {"mfma_64x64x32", 64, 64, 0.925, 4, 55.0},
    {"mfma_128x64x32", 128, 64, 0.94, 3, 119.0},
    {"mfma_64x128x32", 64, 128, 0.945, 3, 109.0},
    {"mfma_32x64x32", 32, 64, 0.85, 6, 25.0},
    {"mfma_64x32x32", 64, 32, 0.85, 6, 25.0},
};
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));
}  // namespace

extern "C" int gemm_f32_variant_count(void) { return kNumVariants; }

extern "C" const char *gemm_f32_variant_name(int variant)
{
    return (variant >= 0 && variant < kNumVariants) ? kVariants[variant].name : nullptr;
}

extern "C" int gemm_f32_choose_variant(int64_t M, int64_t N, int64_t K, int num_cu)
{
    return choose_variant(kVariants, kNumVariants, 0, 0, M, N, K, num_cu);
}

extern "C" int gemm_f32_choose_variant_general(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu)
{
    if ((transa != 0 && transa != 1) || (transb != 0 && transb != 1)) return GEMM_F64_ERR_DIM;
    return choose_variant(kVariants, kNumVariants, transa, transb, M, N, K, num_cu);
}

extern "C" int gemm_f32_ex(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                           int64_t ldb, float *C, int64_t ldc, void *stream, int variant)
{
    return gemm_ex<float>(kVariants, kNumVariants, 0, 0, M, N, K, 1, A, lda, B, ldb, 1, C, ldc, stream, variant);
}

extern "C" int gemm_f32(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb,
                        float *C, int64_t ldc, void *stream)
{
    return gemm_f32_ex(M, N, K, A, lda, B, ldb, C, ldc, stream, -1);
}

extern "C" int gemm_f32_general_ex(int transa, int transb, int64_t M, int64_t N, int64_t K, float alpha, const float *A,
                                   int64_t lda, const float *B, int64_t ldb, float beta, float *C, int64_t ldc,
                                   void *stream, int variant)
{
    return gemm_ex<float>(kVariants, kNumVariants, transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream,
                       variant);
}

extern "C" int gemm_f32_general(int transa, int transb, int64_t M, int64_t N, int64_t K, float alpha, const float *A,
                                int64_t lda, const float *B, int64_t ldb, float beta, float *C, int64_t ldc, void *stream)
{
    return gemm_f32_general_ex(transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream, -1);
}

extern "C" int gemm_f32_general_ws(int transa, int transb, int64_t M, int64_t N, int64_t K, float alpha, const float *A,
                                   int64_t lda, const float *B, int64_t ldb, float beta, float *C, int64_t ldc,
                                   void *workspace, int64_t workspace_bytes, void *stream)
{
    return gemm_ex<float>(kVariants, kNumVariants, transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream, -1,
                       workspace, workspace_bytes);
}

extern "C" int gemm_f32_strided(int64_t M, int64_t N, int64_t K, float alpha, const float *A, int64_t rsa, int64_t csa,
                                const float *B, int64_t rsb, int64_t csb, float beta, float *C, int64_t rsc, int64_t csc,
                                void *stream)
{
    return gemm_strided<float>(kVariants, kNumVariants, M, N, K, alpha, A, rsa, csa, B, rsb, csb, beta, C, rsc, csc, stream);
}

extern "C" int gemm_f32_split_k_plan(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu,
                                     int64_t workspace_bytes, int *variant, int *splits, int *k_chunk)
{
    if ((transa != 0 && transa != 1) || (transb != 0 && transb != 1) || M < 0 || N < 0 || K < 0 || workspace_bytes < 0)
        return GEMM_F64_ERR_DIM;
    if (M > kMaxExtent || N > kMaxExtent || K > kMaxExtent) return GEMM_F64_ERR_TOO_LARGE;
    const Plan plan = plan_split_k(kVariants, kNumVariants, transa, transb, M, N, K, num_cu, (int)sizeof(float), workspace_bytes);
    if (variant) *variant = plan.variant;
    if (splits) *splits = plan.splits;
    if (k_chunk) *k_chunk = plan.k_chunk;
    return GEMM_F64_OK;
}

extern "C" int64_t gemm_f32_split_k_workspace_bytes(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu)
{
    if ((transa != 0 && transa != 1) || (transb != 0 && transb != 1) || M < 0 || N < 0 || K < 0) return 0;
    if (M > kMaxExtent || N > kMaxExtent || K > kMaxExtent) return 0;
    const Plan plan = plan_with_workspace(kVariants, kNumVariants, transa, transb, M, N, K, num_cu, (int)sizeof(float), INT64_MAX);
    return plan_workspace_bytes(kVariants, plan, M, N, (int)sizeof(float));
}

extern "C" int gemm_f32_tail_split_plan(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu, int64_t workspace_bytes,
                                  int *variant, int *tail_tiles, int *tail_splits, int *tail_k_chunk)
{
    if ((transa != 0 && transa != 1) || (transb != 0 && transb != 1) || M < 0 || N < 0 || K < 0 || workspace_bytes < 0)
        return GEMM_F64_ERR_DIM;
    if (M > kMaxExtent || N > kMaxExtent || K > kMaxExtent) return GEMM_F64_ERR_TOO_LARGE;
    const Plan plan = plan_with_workspace(kVariants, kNumVariants, transa, transb, M, N, K, num_cu, (int)sizeof(float), workspace_bytes);
    if (variant) *variant = plan.variant;
    if (tail_tiles) *tail_tiles = plan.splits > 1 ? 0 : plan.tail_tiles;
    if (tail_splits) *tail_splits = plan.splits > 1 ? 1 : plan.tail_splits;
    if (tail_k_chunk) *tail_k_chunk = plan.splits > 1 ? 0 : plan.tail_k_chunk;
    return GEMM_F64_OK;
}
