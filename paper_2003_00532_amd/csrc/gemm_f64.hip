// libgemm_f64.so, double-precision entry points (declared and documented in include/gemm_f64.h).
#include "gemm_host.hpp"

#include <mutex>

using namespace gemm_detail;

namespace {
// Index order is part of the ABI of gemm_f64_ex (tests and the benchmark name variants by index).
// Efficiencies are measured fractions of the FP64 MFMA peak on MI355X: at 8192^3 for the four larger
// tiles (the smaller ones move more bytes per flop through LDS and L2; 64x128 reaches 0.965 on some
// machines of the pool and 0.915 on others, 128x128 the same on all, hence the order), at 2048^3 for
// the two 32-wide tiles, which are only ever chosen for problems of that size or below.
const Variant kVariants[] = {
    {"naive", 0, 0, 0.0, 1, 0.0},
    {"mfma_128x128x16", 128, 128, 0.955, 2, 286.0},
    {"mfma_64x64x16", 64, 64, 0.925, 4, 55.0},
    {"mfma_128x64x16", 128, 64, 0.94, 3, 119.0},
    {"mfma_64x128x16", 64, 128, 0.945, 3, 109.0},
    {"mfma_32x64x16", 32, 64, 0.85, 6, 25.0},
    {"mfma_64x32x16", 64, 32, 0.85, 6, 25.0},
};
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));
}  // namespace

extern "C" int gemm_f64_variant_count(void) { return kNumVariants; }

extern "C" const char *gemm_f64_variant_name(int variant)
{
    return (variant >= 0 && variant < kNumVariants) ? kVariants[variant].name : nullptr;
}

extern "C" int gemm_f64_choose_variant(int64_t M, int64_t N, int64_t K, int num_cu)
{
    return choose_variant(kVariants, kNumVariants, 0, 0, M, N, K, num_cu);
}

extern "C" int gemm_f64_tile_of_block(int64_t block, int64_t tiles_m, int64_t tiles_n, int64_t *tile_m,
                                      int64_t *tile_n)
{
    if (tiles_m < 1 || tiles_n < 1 || tiles_m > INT32_MAX || tiles_n > INT32_MAX || tiles_m * tiles_n > INT32_MAX ||
        block < 0 || block >= tiles_m * tiles_n || !tile_m || !tile_n)
        return GEMM_F64_ERR_DIM;
    uint32_t tm = 0, tn = 0;
    tile_of_block((uint32_t)block, make_tile_map((uint32_t)tiles_m, (uint32_t)tiles_n), tm, tn);
    *tile_m = tm;
    *tile_n = tn;
    return GEMM_F64_OK;
}

extern "C" const char *gemm_f64_strerror(int code)
{
    switch (code) {
    case GEMM_F64_OK: return "success";
    case GEMM_F64_ERR_DIM: return "negative dimension, transpose flag other than 0 or 1, or index out of range";
    case GEMM_F64_ERR_LDA: return "lda smaller than the stored row of A, or a stride of A below 1";
    case GEMM_F64_ERR_LDB: return "ldb smaller than the stored row of B, or a stride of B below 1";
    case GEMM_F64_ERR_LDC: return "ldc smaller than max(1, N), or strides of C below 1 or under which its elements overlap";
    case GEMM_F64_ERR_NULL: return "null pointer for a non-empty operand";
    case GEMM_F64_ERR_ALIGN: return "pointer not aligned to the element size";
    case GEMM_F64_ERR_LAUNCH: return "HIP kernel launch failed";
    case GEMM_F64_ERR_TOO_LARGE: return "dimension exceeds 2^31 - 129";
    case GEMM_F64_ERR_VARIANT: return "unknown kernel variant";
    case GEMM_F64_ERR_SCRATCH:
        return "the split this problem wants needs more than the library's fixed scratch buffer (or the buffer could not be "
               "located on this device); use gemm_f64_general_ws with a workspace of your own";
    default: return "unknown error code";
    }
}

extern "C" int gemm_f64_version(void) { return 500; }

#ifndef GEMM_BUILD_ID
#define GEMM_BUILD_ID "unknown"
#endif
extern "C" const char *gemm_f64_build_id(void)
{
    // the prefix lets the build script find the digest in the file without loading the library
    static const char tagged[] = "gemm-build-id:" GEMM_BUILD_ID;
    return tagged + sizeof("gemm-build-id:") - 1;
}

extern "C" int gemm_f64_choose_variant_general(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu)
{
    if ((transa != 0 && transa != 1) || (transb != 0 && transb != 1)) return GEMM_F64_ERR_DIM;
    return choose_variant(kVariants, kNumVariants, transa, transb, M, N, K, num_cu);
}

extern "C" int gemm_f64_ex(int64_t M, int64_t N, int64_t K, const double *A, int64_t lda, const double *B,
                           int64_t ldb, double *C, int64_t ldc, void *stream, int variant)
{
    return gemm_ex<double>(kVariants, kNumVariants, 0, 0, M, N, K, 1, A, lda, B, ldb, 1, C, ldc, stream, variant);
}

extern "C" int gemm_f64(int64_t M, int64_t N, int64_t K, const double *A, int64_t lda, const double *B, int64_t ldb,
                        double *C, int64_t ldc, void *stream)
{
    return gemm_f64_ex(M, N, K, A, lda, B, ldb, C, ldc, stream, -1);
}

extern "C" int gemm_f64_general_ex(int transa, int transb, int64_t M, int64_t N, int64_t K, double alpha, const double *A,
                                   int64_t lda, const double *B, int64_t ldb, double beta, double *C, int64_t ldc,
                                   void *stream, int variant)
{
    return gemm_ex<double>(kVariants, kNumVariants, transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream,
                       variant);
}

extern "C" int gemm_f64_general(int transa, int transb, int64_t M, int64_t N, int64_t K, double alpha, const double *A,
                                int64_t lda, const double *B, int64_t ldb, double beta, double *C, int64_t ldc, void *stream)
{
    return gemm_f64_general_ex(transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream, -1);
}

extern "C" int gemm_f64_general_ws(int transa, int transb, int64_t M, int64_t N, int64_t K, double alpha, const double *A,
                                   int64_t lda, const double *B, int64_t ldb, double beta, double *C, int64_t ldc,
                                   void *workspace, int64_t workspace_bytes, void *stream)
{
    return gemm_ex<double>(kVariants, kNumVariants, transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream, -1,
                       workspace, workspace_bytes);
}

// ---- the entry point that allocates nothing ---------------------------------------------------------------------
// Scratch for the slabs of a split k range, part of the device image: every GPU the library is loaded on holds its
// own copy at its own address.  In host code the name below is only a handle for hipGetSymbolAddress; the address
// that kernels and copies are given is the one that call returns, looked up once per device.
static __device__ __align__(256) unsigned char scratch[GEMM_F64_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};   // per device, filled on the first call with that device current

// Device address of `scratch` on the current device; nullptr when it cannot be had.
void *scratch_on_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" int gemm_f64_general_static(int transa, int transb, int64_t M, int64_t N, int64_t K, double alpha, const double *A,
                                       int64_t lda, const double *B, int64_t ldb, double beta, double *C, int64_t ldc,
                                       void *stream)
{
    // argument errors first, exactly as the workspace form reports them (nothing is launched for any of them)
    const bool product = (alpha != 0.0) && K != 0;
    const int rc = validate(transa, transb, M, N, K, product, A, lda, B, ldb, C, ldc);
    if (rc != GEMM_F64_OK) return rc;
    if (M == 0 || N == 0 || !product)
        return gemm_ex<double>(kVariants, kNumVariants, transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream, -1);
    // what the rule would like to have when memory is no object
    const Plan plan = plan_with_workspace(kVariants, kNumVariants, transa, transb, M, N, K, current_cu_count(), (int)sizeof(double), INT64_MAX);
    const int64_t wanted = plan_workspace_bytes(kVariants, plan, M, N, (int)sizeof(double));
    if (wanted == 0)
        return gemm_ex<double>(kVariants, kNumVariants, transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream, -1);
    if (wanted > GEMM_F64_STATIC_SCRATCH_BYTES) return GEMM_F64_ERR_SCRATCH;
    void *ptr = scratch_on_current_device();
    if (ptr == nullptr) return GEMM_F64_ERR_SCRATCH;
    return gemm_ex<double>(kVariants, kNumVariants, transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream, -1, ptr,
                           wanted);
}

extern "C" int gemm_f64_strided(int64_t M, int64_t N, int64_t K, double alpha, const double *A, int64_t rsa, int64_t csa,
                                const double *B, int64_t rsb, int64_t csb, double beta, double *C, int64_t rsc, int64_t csc,
                                void *stream)
{
    return gemm_strided<double>(kVariants, kNumVariants, M, N, K, alpha, A, rsa, csa, B, rsb, csb, beta, C, rsc, csc, stream);
}

extern "C" int gemm_f64_strided_path(int64_t M, int64_t N, int64_t K, int64_t rsa, int64_t csa, int64_t rsb, int64_t csb,
                                     int64_t rsc, int64_t csc, int *swapped, int *transa, int *transb, int64_t *lda, int64_t *ldb,
                                     int64_t *ldc, int64_t *es_a, int64_t *es_b, int64_t *es_c)
{
    const int rc = validate_strides(M, N, K, rsa, csa, rsb, csb, rsc, csc);
    if (rc != GEMM_F64_OK) return rc;
    const StridedPath path = strided_path(M, N, K, rsa, csa, rsb, csb, rsc, csc);
    if (swapped) *swapped = path.swapped;
    if (transa) *transa = path.transa;
    if (transb) *transb = path.transb;
    if (lda) *lda = path.lda;
    if (ldb) *ldb = path.ldb;
    if (ldc) *ldc = path.ldc;
    if (es_a) *es_a = path.es_a;
    if (es_b) *es_b = path.es_b;
    if (es_c) *es_c = path.es_c;
    return (int)path.kind;
}

extern "C" int gemm_f64_split_k_plan(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu,
                                     int64_t workspace_bytes, int *variant, int *splits, int *k_chunk)
{
    if ((transa != 0 && transa != 1) || (transb != 0 && transb != 1) || M < 0 || N < 0 || K < 0 || workspace_bytes < 0)
        return GEMM_F64_ERR_DIM;
    if (M > kMaxExtent || N > kMaxExtent || K > kMaxExtent) return GEMM_F64_ERR_TOO_LARGE;
    const Plan plan = plan_split_k(kVariants, kNumVariants, transa, transb, M, N, K, num_cu, (int)sizeof(double), workspace_bytes);
    if (variant) *variant = plan.variant;
    if (splits) *splits = plan.splits;
    if (k_chunk) *k_chunk = plan.k_chunk;
    return GEMM_F64_OK;
}

extern "C" int64_t gemm_f64_split_k_workspace_bytes(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu)
{
    if ((transa != 0 && transa != 1) || (transb != 0 && transb != 1) || M < 0 || N < 0 || K < 0) return 0;
    if (M > kMaxExtent || N > kMaxExtent || K > kMaxExtent) return 0;
    const Plan plan = plan_with_workspace(kVariants, kNumVariants, transa, transb, M, N, K, num_cu, (int)sizeof(double), INT64_MAX);
    return plan_workspace_bytes(kVariants, plan, M, N, (int)sizeof(double));
}

extern "C" int gemm_f64_tail_split_plan(int transa, int transb, int64_t M, int64_t N, int64_t K, int num_cu, int64_t workspace_bytes,
                                  int *variant, int *tail_tiles, int *tail_splits, int *tail_k_chunk)
{
    if ((transa != 0 && transa != 1) || (transb != 0 && transb != 1) || M < 0 || N < 0 || K < 0 || workspace_bytes < 0)
        return GEMM_F64_ERR_DIM;
    if (M > kMaxExtent || N > kMaxExtent || K > kMaxExtent) return GEMM_F64_ERR_TOO_LARGE;
    const Plan plan = plan_with_workspace(kVariants, kNumVariants, transa, transb, M, N, K, num_cu, (int)sizeof(double), workspace_bytes);
    if (variant) *variant = plan.variant;
    if (tail_tiles) *tail_tiles = plan.splits > 1 ? 0 : plan.tail_tiles;
    if (tail_splits) *tail_splits = plan.splits > 1 ? 1 : plan.tail_splits;
    if (tail_k_chunk) *tail_k_chunk = plan.splits > 1 ? 0 : plan.tail_k_chunk;
    return GEMM_F64_OK;
}

extern "C" int gemm_f64_set_epilogue_mode(int mode)
{
    if (mode != kEpilogueAuto && mode != kEpilogueLoadStore && mode != kEpilogueInMemory) return GEMM_F64_ERR_DIM;
    return g_epilogue_mode.exchange(mode);
}

#ifdef GEMM_PHASE_TRACE
// Diagnostic builds only: install (or remove, with NULL) the device buffer the kernels of this file trace into;
// it must hold 8 * (number of workgroups of the launch) 64-bit slots.
extern "C" int gemm_debug_set_trace(void *device_buffer)
{
    unsigned long long *p = static_cast<unsigned long long *>(device_buffer);
    return hipMemcpyToSymbol(HIP_SYMBOL(g_phase_trace), &p, sizeof(p)) == hipSuccess ? 0 : -1;
}
#endif
