// Host side of libgemm_f64.so: argument checks, variant selection, launches.
// The C ABI is declared and documented in include/gemm_f64.h.
#include "../../include/gemm_f64.h"

#include <hip/hip_runtime.h>

#include "gemm_f64_mfma.hpp"

using namespace gemm_f64_detail;

namespace {

struct Variant {
    const char *name;
    int bm, bn;  // macro-tile; 0 for the untiled kernel
    // relative speed of one workgroup's inner loop, per flop, used by the selection model
    double efficiency;
};

// Index order is part of the ABI of gemm_f64_ex (tests and the benchmark name variants by index).
// Efficiencies are measured fractions of the FP64 MFMA peak at 8192^3 on MI355X (the smaller tiles
// move more bytes per flop through LDS and L2; 64x128 and 128x64 fit three workgroups per CU).
const Variant kVariants[] = {
    {"naive", 0, 0, 0.0},
    {"mfma_128x128x16", 128, 128, 0.955},
    {"mfma_64x64x16", 64, 64, 0.915},
    {"mfma_128x64x16", 128, 64, 0.935},
    {"mfma_64x128x16", 64, 128, 0.965},
};
// A compute unit that holds a single workgroup has nothing to run while that workgroup waits at its
// barrier or in its prologue/epilogue (measured: 2048^3 as 256 tiles of 128x128 reaches 80 %).
constexpr double kSingleWorkgroupPenalty = 0.84;
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

template <int BM, int BN, int WM, int WN>
hipError_t launch_mfma(int M, int N, int K, const double *A, int64_t lda, const double *B, int64_t ldb,
                       double *C, int64_t ldc, hipStream_t stream, bool vec)
{
    const int tiles_m = (int)ceil_div(M, BM), tiles_n = (int)ceil_div(N, BN);
    const dim3 grid((unsigned)((int64_t)tiles_m * tiles_n)), block(kThreads);
    // The lean kernel assumes full tiles everywhere, whole K stages and 16-byte-aligned operands.
    const bool lean = vec && (M % BM == 0) && (N % BN == 0) && (K % kBK == 0);
    if (lean)
        hipLaunchKernelGGL((gemm_f64_mfma_kernel<BM, BN, WM, WN, kLean>), grid, block, 0, stream, M, N, K, A, lda, B,
                           ldb, C, ldc, tiles_m, tiles_n, 1);
    else if (vec)
        hipLaunchKernelGGL((gemm_f64_mfma_kernel<BM, BN, WM, WN, kGeneric>), grid, block, 0, stream, M, N, K, A, lda,
                           B, ldb, C, ldc, tiles_m, tiles_n, 1);
    else
        hipLaunchKernelGGL((gemm_f64_mfma_kernel<BM, BN, WM, WN, kStaged>), grid, block, 0, stream, M, N, K, A, lda,
                           B, ldb, C, ldc, tiles_m, tiles_n, 0);
    return hipGetLastError();
}

int validate(int64_t M, int64_t N, int64_t K, const double *A, int64_t lda, const double *B, int64_t ldb,
             const double *C, int64_t ldc)
{
    if (M < 0 || N < 0 || K < 0) return GEMM_F64_ERR_DIM;
    if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX) return GEMM_F64_ERR_TOO_LARGE;
    if (lda < (K > 1 ? K : 1)) return GEMM_F64_ERR_LDA;
    if (ldb < (N > 1 ? N : 1)) return GEMM_F64_ERR_LDB;
    if (ldc < (N > 1 ? N : 1)) return GEMM_F64_ERR_LDC;
    const bool c_live = M > 0 && N > 0;
    const bool ab_live = c_live && K > 0;
    if (c_live && C == nullptr) return GEMM_F64_ERR_NULL;
    if (ab_live && (A == nullptr || B == nullptr)) return GEMM_F64_ERR_NULL;
    if (c_live && ((uintptr_t)C & 7u)) return GEMM_F64_ERR_ALIGN;
    if (ab_live && (((uintptr_t)A & 7u) || ((uintptr_t)B & 7u))) return GEMM_F64_ERR_ALIGN;
    return GEMM_F64_OK;
}

}  // namespace

extern "C" int gemm_f64_variant_count(void) { return kNumVariants; }

extern "C" const char *gemm_f64_variant_name(int variant)
{
    return (variant >= 0 && variant < kNumVariants) ? kVariants[variant].name : nullptr;
}

extern "C" int gemm_f64_choose_variant(int64_t M, int64_t N, int64_t K, int num_cu)
{
    (void)K;
    if (num_cu < 1) num_cu = 1;
    if (M <= 0 || N <= 0) return 1;
    // Tile quantisation model: workgroups are spread over the compute units, so the makespan is
    // about ceil(tiles / CUs) macro-tiles of work per CU; a smaller tile wastes less at the edges
    // and balances better but runs its inner loop a little less efficiently.
    int best = 1;
    double best_cost = 0.0;
    for (int v = 1; v < kNumVariants; ++v) {
        const Variant &var = kVariants[v];
        const int64_t tiles = ceil_div(M, var.bm) * ceil_div(N, var.bn);
        const double eff = var.efficiency * (tiles <= num_cu ? kSingleWorkgroupPenalty : 1.0);
        const double cost = (double)ceil_div(tiles, num_cu) * var.bm * var.bn / eff;
        if (v == 1 || cost < best_cost) {
            best = v;
            best_cost = cost;
        }
    }
    return best;
}

extern "C" int gemm_f64_tile_of_block(int64_t block, int64_t tiles_m, int64_t tiles_n, int64_t *tile_m,
                                      int64_t *tile_n)
{
    if (tiles_m < 1 || tiles_n < 1 || block < 0 || block >= tiles_m * tiles_n || !tile_m || !tile_n)
        return GEMM_F64_ERR_DIM;
    tile_of_block(block, tiles_m, tiles_n, *tile_m, *tile_n);
    return GEMM_F64_OK;
}

extern "C" const char *gemm_f64_strerror(int code)
{
    switch (code) {
    case GEMM_F64_OK: return "success";
    case GEMM_F64_ERR_DIM: return "negative dimension or index out of range";
    case GEMM_F64_ERR_LDA: return "lda smaller than max(1, K)";
    case GEMM_F64_ERR_LDB: return "ldb smaller than max(1, N)";
    case GEMM_F64_ERR_LDC: return "ldc smaller than max(1, N)";
    case GEMM_F64_ERR_NULL: return "null pointer for a non-empty operand";
    case GEMM_F64_ERR_ALIGN: return "pointer not 8-byte aligned";
    case GEMM_F64_ERR_LAUNCH: return "HIP kernel launch failed";
    case GEMM_F64_ERR_TOO_LARGE: return "dimension exceeds 2^31 - 1";
    case GEMM_F64_ERR_VARIANT: return "unknown kernel variant";
    default: return "unknown error code";
    }
}

extern "C" int gemm_f64_version(void) { return 100; }

extern "C" int gemm_f64_ex(int64_t M, int64_t N, int64_t K, const double *A, int64_t lda, const double *B,
                           int64_t ldb, double *C, int64_t ldc, void *stream_, int variant)
{
    const int rc = validate(M, N, K, A, lda, B, ldb, C, ldc);
    if (rc != GEMM_F64_OK) return rc;
    if (variant < -1 || variant >= kNumVariants) return GEMM_F64_ERR_VARIANT;
    if (M == 0 || N == 0 || K == 0) return GEMM_F64_OK;

    hipStream_t stream = (hipStream_t)stream_;
    if (variant == -1) {
        int dev = 0, cus = 256;
        if (hipGetDevice(&dev) == hipSuccess) {
            int v = 0;
            if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cus = v;
        }
        variant = gemm_f64_choose_variant(M, N, K, cus);
    }

    // 16-byte global->LDS loads need aligned operands; their per-lane byte offsets (up to 128 rows of
    // A, 2 rows of B) are 32-bit, which bounds the leading dimensions.
    const bool vec = (((uintptr_t)A | (uintptr_t)B) & 15u) == 0 && (lda % 2 == 0) && (ldb % 2 == 0) &&
                     lda < (1 << 20) && ldb < (1 << 20);
    const int m = (int)M, n = (int)N, k = (int)K;
    hipError_t err = hipSuccess;
    switch (variant) {
    case 0: {
        const int64_t total = M * N;
        const dim3 grid((unsigned)ceil_div(total, 256)), block(256);
        if (ceil_div(total, 256) > INT32_MAX) return GEMM_F64_ERR_TOO_LARGE;
        hipLaunchKernelGGL(gemm_f64_naive_kernel, grid, block, 0, stream, m, n, k, A, lda, B, ldb, C, ldc);
        err = hipGetLastError();
        break;
    }
    case 1: err = launch_mfma<128, 128, 2, 2>(m, n, k, A, lda, B, ldb, C, ldc, stream, vec); break;
    case 2: err = launch_mfma<64, 64, 2, 2>(m, n, k, A, lda, B, ldb, C, ldc, stream, vec); break;
    case 3: err = launch_mfma<128, 64, 2, 2>(m, n, k, A, lda, B, ldb, C, ldc, stream, vec); break;
    case 4: err = launch_mfma<64, 128, 2, 2>(m, n, k, A, lda, B, ldb, C, ldc, stream, vec); break;
    default: return GEMM_F64_ERR_VARIANT;
    }
    return err == hipSuccess ? GEMM_F64_OK : GEMM_F64_ERR_LAUNCH;
}

extern "C" int gemm_f64(int64_t M, int64_t N, int64_t K, const double *A, int64_t lda, const double *B, int64_t ldb,
                        double *C, int64_t ldc, void *stream)
{
    return gemm_f64_ex(M, N, K, A, lda, B, ldb, C, ldc, stream, -1);
}
