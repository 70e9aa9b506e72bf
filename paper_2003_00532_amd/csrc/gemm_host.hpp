// Host side shared by the double and float entry points: argument checks, the tile-quantisation
// model that picks a kernel variant, launches.  The C ABIs are declared in include/gemm_f64.h and
// include/gemm_f32.h; return codes are the GEMM_F64_* values for both.
#pragma once
#include "../../include/gemm_f64.h"

#include <hip/hip_runtime.h>

#include <atomic>

#include "gemm_mfma.hpp"

namespace gemm_detail {

struct Variant {
    const char *name;
    int bm, bn;  // macro-tile; 0 for the untiled kernel
    // measured fraction of the MFMA peak reached by this tile shape when every compute unit holds as
    // many of its workgroups as fit, used by the selection model
    double efficiency;
    int resident;  // workgroups of this shape that fit on one compute unit (registers and LDS decide)
    // MFMA issue slots per tile that its prologue and epilogue cost beyond the K loop when the compute
    // units are full (fitted on 16384^2 x 256, checked on 6144^2 x 1024 and 1024 x 8192 x 512)
    double overhead;
};

// With fewer workgroups on a compute unit than fit, there are fewer waves to run while one waits at its
// barrier or in its prologue/epilogue.  Measured at 2048^3 in double: one resident workgroup of 128x128
// reaches 0.84 of what two do; two of 64x128 reach 0.92 of what three do.
inline double few_resident_penalty(int resident_now, int resident_full)
{
    if (resident_now >= resident_full) return 1.0;
    return resident_now <= 1 ? 0.84 : resident_now == 2 ? 0.92 : 0.96;
}

// What a tile costs besides its MFMAs when it runs on its own (fetching the first stages, reading and
// writing C), in MFMA issue slots; it only matters for problems of a few tiles.
constexpr double kLoneTileSlots = 96.0;

// What a launch costs once, whatever its length: at its start every workgroup is in its prologue and at its end the
// last ones are in their epilogues with nothing to hide under, and both grow with the outputs of a tile.  In MFMA issue
// slots per 4096 outputs of a tile (64 x 64: 8 us in double).  Fitted on the measured table of every variant on 17
// shapes (ten tables from three machines and both precisions): the mean regret of the choice falls from 1.3 % to 0.4 %,
// the largest from 15 % to 6 %, and the fit is flat from 250 to 600.
constexpr double kLaunchExposureSlots = 300.0;
inline double launch_exposure(const Variant &var) { return kLaunchExposureSlots * (double)(var.bm * var.bn) / 4096.0; }

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Grid of the element-wise kernels (256 threads a block, each striding over the elements): one block per 256 elements
// up to 2^22 blocks; the runtime refuses launches of 2^32 threads or more, and C may well have more elements.
inline unsigned elementwise_blocks(int64_t elements)
{
    const int64_t blocks = ceil_div(elements, 256), cap = (int64_t)1 << 22;
    return (unsigned)(blocks < cap ? blocks : cap);
}

// A 32-wide panel exists only for an operand whose k index is contiguous in memory (A as given, B
// stored transposed), so the 32-row variants need transa == 0 and the 32-column ones transb == 1.
inline bool variant_available(const Variant &v, int transa, int transb)
{
    if (v.bm == 32 && transa) return false;
    if (v.bn == 32 && !transb) return false;
    return true;
}

// Selection model, in units of one MFMA issue slot of a SIMD (64 cycles in double).  A macro-tile costs
// each of its four waves (BM/32) * (BN/32) MFMAs per k-step at the variant's measured efficiency, plus
// what is not hidden of its prologue and epilogue (a measured number of slots per variant: it grows with
// the outputs per tile and is larger where fewer workgroups share a compute unit).  Workgroups are spread over the compute
// units, so the throughput-bound makespan is ceil(tiles / CUs) such tiles, plus what the start and the end of a launch
// expose (launch_exposure): a smaller tile wastes less at the edges, balances better and exposes less, but runs its
// inner loop a little less efficiently.  The makespan cannot
// be shorter than the time one tile needs on its own (the MFMA chain of one wave plus a fixed start-up
// and write-back cost): that floor is what counts when there are fewer tiles than compute units.
// Variant 0 (untiled) is never chosen.
inline double variant_cost(const Variant &var, int64_t M, int64_t N, int64_t K, int64_t slices, int num_cu)
{
    const double ksteps = (double)ceil_div(K, 4);
    const int64_t tiles = ceil_div(M, var.bm) * ceil_div(N, var.bn) * slices;
    const int64_t per_cu = ceil_div(tiles, num_cu);
    const double eff = var.efficiency * few_resident_penalty(per_cu < var.resident ? (int)per_cu : var.resident, var.resident);
    const double wave_chain = (double)(var.bm / 32) * (var.bn / 32);   // MFMAs per k-step in one wave
    const double throughput = (double)per_cu * (wave_chain * ksteps / eff + var.overhead) + launch_exposure(var);
    const double floor_alone = wave_chain * ksteps + kLoneTileSlots;
    return throughput > floor_alone ? throughput : floor_alone;
}

inline int choose_variant(const Variant *variants, int count, int transa, int transb, int64_t M, int64_t N, int64_t K,
                          int num_cu, int64_t slices = 1, double *cost_out = nullptr)
{
    if (num_cu < 1) num_cu = 1;
    if (K < 1) K = 1;
    int best = 1;
    double best_cost = 0.0;
    if (M > 0 && N > 0)
        for (int v = 1; v < count; ++v) {
            if (!variant_available(variants[v], transa, transb)) continue;
            const double cost = variant_cost(variants[v], M, N, K, slices, num_cu);
            if (v == 1 || cost < best_cost) {
                best = v;
                best_cost = cost;
            }
        }
    if (cost_out) *cost_out = best_cost;
    return best;
}

// Split K.  A problem of few tiles and a long k range leaves most compute units idle while each tile
// walks its whole range; cutting the range into S slices gives S times as many workgroups of a S-th of
// the length, at the price of S output slabs in a workspace and a second, memory-bound step that adds
// them up (in a fixed order: the result does not depend on scheduling).  The plan is a pure function
// of the shape, the CU count and the workspace on offer: for each S the cost of the first step by the
// model above, plus the second step as (S + 2) M N elements moved at about 2.5 TB/s and a launch of 4 us,
// converted to the model's unit (more than twice what the second step measures, which is the margin: of eighteen
// shapes of few tiles ten get a plan this way, of which nine gain, up to a factor of two, and one is even).
struct Plan {
    int variant;
    int splits;     // 1: no split
    int k_chunk;    // slice length, a multiple of the stage depth (K itself when splits == 1)
    // Tail split (splits == 1 only): the last tail_tiles tiles of the grouped order are computed in tail_splits
    // slices of tail_k_chunk each; 0 tiles: none.
    int tail_tiles = 0, tail_splits = 1, tail_k_chunk = 0;
};

// Bytes of workspace a plan uses.
inline int64_t plan_workspace_bytes(const Variant *variants, const Plan &p, int64_t M, int64_t N, int elem_bytes)
{
    if (p.splits > 1) return (int64_t)p.splits * M * N * elem_bytes;
    if (p.tail_tiles > 0) return (int64_t)p.tail_tiles * p.tail_splits * variants[p.variant].bm * variants[p.variant].bn * elem_bytes;
    return 0;
}

inline Plan plan_split_k(const Variant *variants, int count, int transa, int transb, int64_t M, int64_t N, int64_t K,
                         int num_cu, int elem_bytes, int64_t workspace_bytes)
{
    double base_cost = 0.0;
    Plan best{choose_variant(variants, count, transa, transb, M, N, K, num_cu, 1, &base_cost), 1, (int)K};
    if (M <= 0 || N <= 0 || K <= 0) return best;
    const int bk = 8 * (16 / elem_bytes);
    const double slot_seconds = (elem_bytes == 8 ? 64.0 : 32.0) / 2.4e9;
    double best_cost = base_cost;
    static const int candidates[] = {2, 3, 4, 5, 6, 8, 10, 12, 16, 24, 32};
    for (int s : candidates) {
        const int64_t chunk = ceil_div(ceil_div(K, s), bk) * bk;
        const int64_t slices = ceil_div(K, chunk);
        if (slices < 2 || slices * M * N * elem_bytes > workspace_bytes) continue;
        double cost = 0.0;
        const int v = choose_variant(variants, count, transa, transb, M, N, chunk, num_cu, slices, &cost);
        cost += ((double)(slices + 2) * M * N * elem_bytes / 2.5e12 + 4e-6) / slot_seconds;
        if (cost < best_cost) {
            best_cost = cost;
            best = Plan{v, (int)slices, (int)chunk};
        }
    }
    return best;
}

// The kernels hold extents and tile origins in 32-bit integers and form "origin + tile size" and "extent + stage
// depth - 1" in them; the largest tile is 128 wide and the deepest stage 32, so extents up to 2^31 - 1 - 128 are safe.
constexpr int64_t kMaxExtent = (int64_t)INT32_MAX - 128;

// Tail split.  Workgroups are dispatched in rounds of (compute units x resident workgroups) slots; when the tiles of
// a problem make up some whole rounds and a small rest, the rest occupies a few compute units for the time of a whole
// tile while the others idle (2088 x 2049 x 2047 with 64 x 64 tiles: 1089 tiles on 1024 slots, the last 65 tiles run
// alone).  With a workspace the k range of just those last tiles is cut into S slices so that tail * S units fill one
// round of slots, each a fraction 1/S of a tile long; their slabs are added in a second, small launch.  The plan prices
// every variant that way with the model of variant_cost and keeps the cheapest if it beats the unsplit choice (the second
// step is priced at more than twice what it measures, which is margin enough: of fifteen shapes with partial rounds the nine
// that get a plan this way all gain, 1.2 to 9 points of the peak).
inline Plan plan_tail_split(const Variant *variants, int count, int transa, int transb, int64_t M, int64_t N, int64_t K,
                            int num_cu, int elem_bytes, int64_t workspace_bytes, const Plan &unsplit, double unsplit_cost)
{
    Plan best = unsplit;
    if (M <= 0 || N <= 0 || K <= 0 || workspace_bytes <= 0) return best;
    const int bk = 8 * (16 / elem_bytes);
    const double slot_seconds = (elem_bytes == 8 ? 64.0 : 32.0) / 2.4e9;
    double best_cost = unsplit_cost;
    const int64_t nk = ceil_div(K, bk);
    for (int v = 1; v < count; ++v) {
        const Variant &var = variants[v];
        if (!variant_available(var, transa, transb)) continue;
        const int64_t tiles = ceil_div(M, var.bm) * ceil_div(N, var.bn);
        const int64_t slots = (int64_t)num_cu * var.resident;
        if (tiles <= slots || tiles > INT32_MAX) continue;   // fewer tiles than slots is the business of split K
        const int64_t rounds = tiles / slots, tail = tiles % slots;
        if (tail == 0) continue;
        int64_t s = slots / tail;
        if (s > 32) s = 32;
        if (s > nk) s = nk;
        if (s < 2) continue;
        const int64_t chunk_stages = ceil_div(nk, s);
        const int64_t slices = ceil_div(nk, chunk_stages);
        if (slices < 2) continue;
        const int64_t bytes = tail * slices * var.bm * var.bn * elem_bytes;
        if (bytes > workspace_bytes) continue;
        const double wave_chain = (double)(var.bm / 32) * (var.bn / 32);
        const double tile_cost = wave_chain * (double)ceil_div(K, 4) / var.efficiency + var.overhead;
        const double unit_cost = wave_chain * (double)(chunk_stages * bk / 4) / var.efficiency + var.overhead;
        const double reduce = ((double)(slices + 2) * tail * var.bm * var.bn * elem_bytes / 2.5e12 + 4e-6) / slot_seconds;
        const double cost = (double)(rounds * var.resident) * tile_cost + (double)ceil_div(tail * slices, num_cu) * unit_cost + reduce +
                            0.5 * launch_exposure(var);   // the start only: the end of such a launch is its short units
        if (cost < best_cost) {
            best_cost = cost;
            best = Plan{v, 1, (int)K, (int)tail, (int)slices, (int)(chunk_stages * bk)};
        }
    }
    return best;
}

// What a call with a workspace on offer does: split K, or a tail split, or neither.
inline Plan plan_with_workspace(const Variant *variants, int count, int transa, int transb, int64_t M, int64_t N, int64_t K,
                                int num_cu, int elem_bytes, int64_t workspace_bytes)
{
    const Plan split = plan_split_k(variants, count, transa, transb, M, N, K, num_cu, elem_bytes, workspace_bytes);
    if (split.splits > 1) return split;
    double cost = 0.0;
    choose_variant(variants, count, transa, transb, M, N, K < 1 ? 1 : K, num_cu, 1, &cost);
    return plan_tail_split(variants, count, transa, transb, M, N, K, num_cu, elem_bytes, workspace_bytes, split, cost);
}

// Stored shapes: A is M x K (K x M when transa), B is K x N (N x K when transb), C is M x N; a leading
// dimension must cover the stored row.  A and B are only required when the product is formed
// (ab_read: alpha != 0 and K > 0).
template <typename T>
int validate(int transa, int transb, int64_t M, int64_t N, int64_t K, bool ab_read, const T *A, int64_t lda, const T *B,
             int64_t ldb, const T *C, int64_t ldc)
{
    if (M < 0 || N < 0 || K < 0) return GEMM_F64_ERR_DIM;
    if ((transa != 0 && transa != 1) || (transb != 0 && transb != 1)) return GEMM_F64_ERR_DIM;
    if (M > kMaxExtent || N > kMaxExtent || K > kMaxExtent) return GEMM_F64_ERR_TOO_LARGE;
    const int64_t a_width = transa ? M : K, b_width = transb ? K : N;
    if (lda < (a_width > 1 ? a_width : 1)) return GEMM_F64_ERR_LDA;
    if (ldb < (b_width > 1 ? b_width : 1)) return GEMM_F64_ERR_LDB;
    if (ldc < (N > 1 ? N : 1)) return GEMM_F64_ERR_LDC;
    const bool c_live = M > 0 && N > 0;
    const bool ab_live = c_live && K > 0 && ab_read;
    if (c_live && C == nullptr) return GEMM_F64_ERR_NULL;
    if (ab_live && (A == nullptr || B == nullptr)) return GEMM_F64_ERR_NULL;
    const uintptr_t mask = sizeof(T) - 1;
    if (c_live && ((uintptr_t)C & mask)) return GEMM_F64_ERR_ALIGN;
    if (ab_live && (((uintptr_t)A & mask) || ((uintptr_t)B & mask))) return GEMM_F64_ERR_ALIGN;
    return GEMM_F64_OK;
}

// The 16-byte global->LDS copies take any address that is aligned to the element (measured: an 8-byte
// aligned double operand with an odd leading dimension is copied correctly and at nearly full speed), so
// alignment never decides the path.  What does is the 32-bit per-lane byte offset of those copies, which
// spans up to 128 stored rows: the leading dimensions must stay below 2^32 / (128 * sizeof(T)).
template <typename T>
bool async_copies_possible(int64_t lda, int64_t ldb)
{
    constexpr int64_t limit = ((int64_t)1 << 32) / (128 * (int64_t)sizeof(T));
    return lda < limit && ldb < limit;
}

// One product to launch: the operands as the caller stores them, and how the k range is sliced.
template <typename T>
struct Job {
    int transa, transb;
    int M, N, K;
    T alpha;
    const T *A;
    int64_t lda;
    const T *B;
    int64_t ldb;
    T beta;
    T *C;
    int64_t ldc;
    hipStream_t stream;
    int slices;     // grid height
    SplitK split;
    // Sampled operands: elements es.a / es.b apart along the contiguous index, or leading dimensions that do not
    // cover a row; such a job runs in the kSampled mode (64 x 64 tile only) whatever its other properties.
    bool sampled = false;
    ElemStrides es{1, 1, 1};
    // Tail split: the last tail_tiles tiles of the grouped order in tail_splits slices of tail_k_chunk, into `slabs`
    int tail_tiles = 0, tail_splits = 1, tail_k_chunk = 0;
    T *slabs = nullptr;
};

template <typename T, int BM, int BN, int WM, int WN, bool TA, bool TB>
hipError_t launch_mfma_t(const Job<T> &j)
{
    constexpr int BK = 8 * (16 / (int)sizeof(T));
    const int tiles_m = (int)ceil_div(j.M, BM), tiles_n = (int)ceil_div(j.N, BN);
    const int64_t tiles = (int64_t)tiles_m * tiles_n;
    const bool vec = async_copies_possible<T>(j.lda, j.ldb);
    // The lean kernel assumes full tiles everywhere and whole K stages (in every slice).
    const bool lean = !j.sampled && vec && (j.M % BM == 0) && (j.N % BN == 0) && (j.K % BK == 0) && (j.split.k_chunk % BK == 0) &&
                      (j.tail_k_chunk % BK == 0);
    const int64_t whole = tiles - j.tail_tiles;   // tiles computed over the whole k range, one block each
    const dim3 grid((unsigned)(whole + (int64_t)j.tail_tiles * j.tail_splits), (unsigned)j.slices), block(kThreads);
    const TileMap map = make_tile_map((uint32_t)tiles_m, (uint32_t)tiles_n, (uint32_t)whole);
    TailSplit tail = no_tail();
    if (j.tail_tiles > 0)
        tail = TailSplit{(uint32_t)whole, make_fast_div((uint32_t)j.tail_splits), j.tail_k_chunk,
                         j.transa ? (int64_t)j.tail_k_chunk * j.lda : (int64_t)j.tail_k_chunk,
                         j.transb ? (int64_t)j.tail_k_chunk : (int64_t)j.tail_k_chunk * j.ldb, j.slabs};
    if (j.sampled) {
        // built for one tile shape only (the mode needs more registers than the largest tile leaves)
        if constexpr (BM == 64 && BN == 64) {
            hipLaunchKernelGGL((gemm_mfma_kernel<T, BM, BN, WM, WN, kSampled, TA, TB>), grid, block, 0, j.stream, j.M, j.N, j.K,
                               j.alpha, j.A, j.lda, j.B, j.ldb, j.beta, j.C, j.ldc, map, j.split, j.es, tail);
            return hipGetLastError();
        } else {
            return hipErrorInvalidValue;
        }
    }
    if (lean)
        hipLaunchKernelGGL((gemm_mfma_kernel<T, BM, BN, WM, WN, kLean, TA, TB>), grid, block, 0, j.stream, j.M, j.N, j.K,
                           j.alpha, j.A, j.lda, j.B, j.ldb, j.beta, j.C, j.ldc, map, j.split, j.es, tail);
    else if (vec)
        hipLaunchKernelGGL((gemm_mfma_kernel<T, BM, BN, WM, WN, kGeneric, TA, TB>), grid, block, 0, j.stream, j.M, j.N, j.K,
                           j.alpha, j.A, j.lda, j.B, j.ldb, j.beta, j.C, j.ldc, map, j.split, j.es, tail);
    else
        hipLaunchKernelGGL((gemm_mfma_kernel<T, BM, BN, WM, WN, kStaged, TA, TB>), grid, block, 0, j.stream, j.M, j.N, j.K,
                           j.alpha, j.A, j.lda, j.B, j.ldb, j.beta, j.C, j.ldc, map, j.split, j.es, tail);
    return hipGetLastError();
}

template <typename T, int BM, int BN, int WM, int WN>
hipError_t launch_mfma(const Job<T> &j)
{
    if (!j.transa && !j.transb) return launch_mfma_t<T, BM, BN, WM, WN, false, false>(j);
    if (!j.transa && j.transb) return launch_mfma_t<T, BM, BN, WM, WN, false, true>(j);
    if (j.transa && !j.transb) return launch_mfma_t<T, BM, BN, WM, WN, true, false>(j);
    return launch_mfma_t<T, BM, BN, WM, WN, true, true>(j);
}

template <typename T>
hipError_t launch_variant(int variant, const Job<T> &j)
{
    switch (variant) {
    case 1: return launch_mfma<T, 128, 128, 2, 2>(j);
    case 2: return launch_mfma<T, 64, 64, 2, 2>(j);
    case 3: return launch_mfma<T, 128, 64, 2, 2>(j);
    case 4: return launch_mfma<T, 64, 128, 2, 2>(j);
    case 5:  // 32-row tiles: A must be k-contiguous
        return j.transb ? launch_mfma_t<T, 32, 64, 2, 2, false, true>(j) : launch_mfma_t<T, 32, 64, 2, 2, false, false>(j);
    case 6:  // 32-column tiles: B must be k-contiguous
        return j.transa ? launch_mfma_t<T, 64, 32, 2, 2, true, true>(j) : launch_mfma_t<T, 64, 32, 2, 2, false, true>(j);
    default: return hipErrorInvalidValue;
    }
}

template <typename T>
hipError_t launch_naive(const Job<T> &j)
{
    const dim3 grid(elementwise_blocks((int64_t)j.M * j.N)), block(256);
    hipLaunchKernelGGL(gemm_naive_kernel<T>, grid, block, 0, j.stream, j.M, j.N, j.K, j.alpha, j.A, j.transa ? 1 : j.lda,
                       j.transa ? j.lda : 1, j.B, j.transb ? 1 : j.ldb, j.transb ? j.ldb : 1, j.beta, j.C, j.ldc, (int64_t)1);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_scale(int M, int N, T beta, T *C, int64_t rsc, int64_t csc, hipStream_t stream)
{
    const dim3 grid(elementwise_blocks((int64_t)M * N)), block(256);
    hipLaunchKernelGGL(scale_c_kernel<T>, grid, block, 0, stream, M, N, beta, C, rsc, csc);
    return hipGetLastError();
}

// How C is updated when alpha == beta == 1 (the paper's own operation).  Either each lane loads its elements, adds
// and stores; or it hands its sums to the memory system as floating-point additions performed at the L2 cache
// (global_atomic_add_f64 without return).  Every element of C belongs to exactly one lane, so the second form is the
// same single rounding of c + s and the result is the same bits (tested on the device against the first form, special
// values included); what differs is that the wave does not wait for C to arrive, so its registers and LDS are free for
// the next workgroup one memory latency earlier.  Measured at 16384^2 x K: K = 256 2.32 -> 2.22 ms, K = 512 4.24 ->
// 4.12 ms, K = 1024 8.06 -> 7.96 ms; but K = 128 1.42 -> 1.77 ms, because the additions themselves take 1.64 ms for
// 16384^2 elements (load and store: 0.88 ms) and must fit under the MFMA time, which they do from K = 242 upwards.
// Hardware floating-point additions in memory are only defined for ordinary device memory (not for host memory
// mapped into the device, nor managed memory) and are only used on the memory of the GPU that runs the kernel, so the
// owner of C is asked first; single precision keeps the first
// form (its additions in memory do not honour denormals).
enum { kEpilogueAuto = 0, kEpilogueLoadStore = 1, kEpilogueInMemory = 2 };
inline std::atomic<int> g_epilogue_mode{kEpilogueAuto};   // a diagnostic switch, see gemm_f64_set_epilogue_mode

template <typename T>
bool accumulate_in_memory(int64_t M, int64_t N, int64_t K, T alpha, T beta, const T *C)
{
    if (!std::is_same<T, double>::value || alpha != T(1) || beta != T(1)) return false;
    const int mode = g_epilogue_mode.load(std::memory_order_relaxed);
    if (mode == kEpilogueLoadStore) return false;
    if (mode == kEpilogueAuto && (K < 256 || M * N < ((int64_t)1 << 20))) return false;
    hipPointerAttribute_t attr;
    int dev = -1;
    if (hipPointerGetAttributes(&attr, C) != hipSuccess || hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    // the memory of the device that runs the kernel: additions sent to a peer's memory cross a link that need not
    // carry them
    return attr.type == hipMemoryTypeDevice && attr.device == dev;
}

inline int current_cu_count()
{
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
        return v;
    return 256;
}

// The body common to all entry points: C <- alpha * op(A) op(B) + beta * C.
//   alpha == 0 or K == 0: A and B are not read; C is scaled by beta (untouched when beta == 1).
//   beta == 0: C is not read.
// With a workspace (device memory, may be null) and variant == -1 the k range may be split, see plan_split_k.
template <typename T>
int gemm_ex(const Variant *variants, int count, int transa, int transb, int64_t M, int64_t N, int64_t K, T alpha,
            const T *A, int64_t lda, const T *B, int64_t ldb, T beta, T *C, int64_t ldc, void *stream_, int variant,
            void *workspace = nullptr, int64_t workspace_bytes = 0)
{
    const bool product = (alpha != T(0)) && K != 0;
    const int rc = validate(transa, transb, M, N, K, product, A, lda, B, ldb, C, ldc);
    if (rc != GEMM_F64_OK) return rc;
    if (variant < -1 || variant >= count) return GEMM_F64_ERR_VARIANT;
    if (workspace_bytes < 0 || (workspace_bytes > 0 && workspace == nullptr)) return GEMM_F64_ERR_NULL;
    if (workspace && ((uintptr_t)workspace & (sizeof(T) - 1))) return GEMM_F64_ERR_ALIGN;
    if (M == 0 || N == 0) return GEMM_F64_OK;
    if (ceil_div(M * N, 256) > INT32_MAX) return GEMM_F64_ERR_TOO_LARGE;
    hipStream_t stream = (hipStream_t)stream_;
    const int m = (int)M, n = (int)N, k = (int)K;
    (void)hipGetLastError();   // an error left behind by an earlier, unrelated call must not be reported as this launch's
    hipError_t err = hipSuccess;
    if (!product) {
        if (beta == T(1)) return GEMM_F64_OK;
        err = launch_scale<T>(m, n, beta, C, ldc, 1, stream);
        return err == hipSuccess ? GEMM_F64_OK : GEMM_F64_ERR_LAUNCH;
    }
    Job<T> job{transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, stream, 1, SplitK{k, 0, 0, 0}};
    job.split.flags = accumulate_in_memory<T>(M, N, K, alpha, beta, C) ? kFlagAtomicC : 0;
    if (variant == -1) {
        const Plan plan = plan_with_workspace(variants, count, transa, transb, M, N, K, current_cu_count(), (int)sizeof(T),
                                              workspace ? workspace_bytes : 0);
        variant = plan.variant;
        if (plan.splits > 1) {
            // first step: slice y of the k range into slab y of the workspace (dense M x N), nothing scaled yet
            T *slabs = static_cast<T *>(workspace);
            job.alpha = T(1);
            job.beta = T(0);
            job.C = slabs;
            job.ldc = N;
            job.slices = plan.splits;
            job.split = SplitK{plan.k_chunk, transa ? (int64_t)plan.k_chunk * lda : (int64_t)plan.k_chunk,
                               transb ? (int64_t)plan.k_chunk : (int64_t)plan.k_chunk * ldb, M * N};
            err = launch_variant<T>(variant, job);
            if (err != hipSuccess) return GEMM_F64_ERR_LAUNCH;
            // second step: C <- alpha * (sum of the slabs, in order) + beta * C
            const dim3 grid(elementwise_blocks(M * N)), block(256);
            hipLaunchKernelGGL(split_k_reduce_kernel<T>, grid, block, 0, stream, m, n, plan.splits, alpha, slabs, beta, C, ldc);
            return hipGetLastError() == hipSuccess ? GEMM_F64_OK : GEMM_F64_ERR_LAUNCH;
        }
        if (plan.tail_tiles > 0) {
            // one launch computes the tiles of the whole rounds into C and the last tiles, in slices, into slabs of the
            // workspace; a second, small one adds each tile's slabs in order and applies alpha and beta
            const Variant &var = variants[variant];
            T *slabs = static_cast<T *>(workspace);
            job.tail_tiles = plan.tail_tiles;
            job.tail_splits = plan.tail_splits;
            job.tail_k_chunk = plan.tail_k_chunk;
            job.slabs = slabs;
            err = launch_variant<T>(variant, job);
            if (err != hipSuccess) return GEMM_F64_ERR_LAUNCH;
            const uint32_t tiles_m = (uint32_t)ceil_div(M, var.bm), tiles_n = (uint32_t)ceil_div(N, var.bn);
            const uint32_t whole = tiles_m * tiles_n - (uint32_t)plan.tail_tiles;
            const dim3 grid((unsigned)((int64_t)plan.tail_tiles * (var.bm * var.bn / 256))), block(256);
            hipLaunchKernelGGL(tail_reduce_kernel<T>, grid, block, 0, stream, m, n, var.bm, var.bn,
                               make_tile_map(tiles_m, tiles_n, whole), whole, plan.tail_splits, alpha, slabs, beta, C, ldc);
            return hipGetLastError() == hipSuccess ? GEMM_F64_OK : GEMM_F64_ERR_LAUNCH;
        }
    } else if (variant > 0 && !variant_available(variants[variant], transa, transb)) {
        return GEMM_F64_ERR_VARIANT;
    }
    err = variant == 0 ? launch_naive<T>(job) : launch_variant<T>(variant, job);
    return err == hipSuccess ? GEMM_F64_OK : GEMM_F64_ERR_LAUNCH;
}

// How one operand with two strides maps onto the row-major kernels.  kRows: the column stride is 1 and the row
// stride is a leading dimension that covers the row; kColumns: the row stride is 1 and the column stride covers
// the column (the transposed view of a row-major array); kNeither: anything else (sampled sub-matrices, rows that
// share elements), which the tiled kernel handles in its kSampled mode.  An extent of 0 or 1 makes its stride
// irrelevant.
enum Layout { kRows, kColumns, kNeither };

inline Layout classify(int64_t rows, int64_t cols, int64_t rs, int64_t cs, int64_t *ld)
{
    if ((cs == 1 || cols <= 1) && (rs >= cols || rows <= 1)) {
        *ld = rows <= 1 ? (cols > 1 ? cols : 1) : rs;
        return kRows;
    }
    if ((rs == 1 || rows <= 1) && (cs >= rows || cols <= 1)) {
        *ld = cols <= 1 ? (rows > 1 ? rows : 1) : cs;
        return kColumns;
    }
    return kNeither;
}

// C <- alpha * A B + beta * C with X(r, c) = X[r * rs + c * cs] for each operand (Section 2.9: an operand is an
// index space plus an affine layout map; Section 2.15 Q4: strides and transposes are such maps).  When every
// operand has a unit stride the call is the transposed signature (a column-major C is the transposed problem
// C^T = B^T A^T, which sums the same products in the same order); otherwise the same tiled kernel runs in its
// kSampled mode.  The elements of C must be distinct: one of its strides must span the whole extent of the other.
// What a strided call becomes.  kTransposed: the transposed-signature call on the tiled kernels.  kSampled: the tiled
// kernels in their kSampled mode, because some operand has no unit stride or no leading dimension that covers its
// rows (es_a / es_b / es_c are the element strides along the index the kernel treats as contiguous).  When C is
// column-major, or its row stride is the smaller one, the transposed problem C^T = B^T A^T is what runs (swapped),
// and every field describes that call as issued.
struct StridedPath {
    enum Kind { kTransposed = 1, kSampled = 2 } kind;
    bool swapped;
    int transa, transb;
    int64_t lda, ldb, ldc;
    int64_t es_a, es_b, es_c;
};

// Validation of the strides alone (what needs no pointers), shared by the entry point and the host-side query.
inline int validate_strides(int64_t M, int64_t N, int64_t K, int64_t rsa, int64_t csa, int64_t rsb, int64_t csb, int64_t rsc,
                            int64_t csc)
{
    if (M < 0 || N < 0 || K < 0) return GEMM_F64_ERR_DIM;
    if (M > kMaxExtent || N > kMaxExtent || K > kMaxExtent) return GEMM_F64_ERR_TOO_LARGE;
    if (rsa < 1 || csa < 1) return GEMM_F64_ERR_LDA;
    if (rsb < 1 || csb < 1) return GEMM_F64_ERR_LDB;
    if (rsc < 1 || csc < 1) return GEMM_F64_ERR_LDC;
    if (M > 1 && N > 1) {
        const __int128 row_span = (__int128)csc * (N - 1) + 1, col_span = (__int128)rsc * (M - 1) + 1;
        if (!((__int128)rsc >= row_span || (__int128)csc >= col_span)) return GEMM_F64_ERR_LDC;
    }
    return GEMM_F64_OK;
}

inline StridedPath strided_path(int64_t M, int64_t N, int64_t K, int64_t rsa, int64_t csa, int64_t rsb, int64_t csb,
                                int64_t rsc, int64_t csc)
{
    StridedPath p{StridedPath::kSampled, false, 0, 0, 1, 1, 1, 1, 1, 1};
    const Layout lc = classify(M, N, rsc, csc, &p.ldc);
    if (lc == kNeither) {   // the output of the problem that runs sits at O[r * ldc + c * es_c]: columns along the smaller stride
        p.swapped = rsc < csc;
        p.ldc = p.swapped ? csc : rsc;
        p.es_c = p.swapped ? rsc : csc;
    } else {
        p.swapped = lc == kColumns;
    }
    // first operand F (rows x K) and second operand S (K x cols) of the problem that runs: A and B, or, swapped,
    // B^T and A^T (C^T = B^T A^T; transposing an operand swaps its two strides)
    const int64_t rows = p.swapped ? N : M, cols = p.swapped ? M : N;
    const int64_t rsf = p.swapped ? csb : rsa, csf = p.swapped ? rsb : csa;
    const int64_t rss = p.swapped ? csa : rsb, css = p.swapped ? rsa : csb;
    const Layout lf = classify(rows, K, rsf, csf, &p.lda), ls = classify(K, cols, rss, css, &p.ldb);
    p.transa = lf == kColumns;
    p.transb = ls == kColumns;
    if (lf != kNeither && ls != kNeither && lc != kNeither) {
        p.kind = StridedPath::kTransposed;
        return p;
    }
    if (lf == kNeither) {   // F(x, k) = F[x * rsf + k * csf]: treat the direction of the smaller stride as contiguous
        p.transa = csf > rsf;
        p.lda = p.transa ? csf : rsf;
        p.es_a = p.transa ? rsf : csf;
    }
    if (ls == kNeither) {   // S(k, x) = S[k * rss + x * css]
        p.transb = rss <= css;
        p.ldb = p.transb ? css : rss;
        p.es_b = p.transb ? rss : css;
    }
    return p;
}

template <typename T>
int gemm_strided(const Variant *variants, int count, int64_t M, int64_t N, int64_t K, T alpha, const T *A, int64_t rsa,
                 int64_t csa, const T *B, int64_t rsb, int64_t csb, T beta, T *C, int64_t rsc, int64_t csc, void *stream_)
{
    const int rc = validate_strides(M, N, K, rsa, csa, rsb, csb, rsc, csc);
    if (rc != GEMM_F64_OK) return rc;
    const bool product = (alpha != T(0)) && K != 0;
    const bool c_live = M > 0 && N > 0, ab_live = c_live && product;
    if (c_live && C == nullptr) return GEMM_F64_ERR_NULL;
    if (ab_live && (A == nullptr || B == nullptr)) return GEMM_F64_ERR_NULL;
    const uintptr_t mask = sizeof(T) - 1;
    if (c_live && ((uintptr_t)C & mask)) return GEMM_F64_ERR_ALIGN;
    if (ab_live && (((uintptr_t)A & mask) || ((uintptr_t)B & mask))) return GEMM_F64_ERR_ALIGN;
    if (!c_live) return GEMM_F64_OK;
    if (ceil_div(M * N, 256) > INT32_MAX) return GEMM_F64_ERR_TOO_LARGE;

    const StridedPath path = strided_path(M, N, K, rsa, csa, rsb, csb, rsc, csc);
    const T *F = path.swapped ? B : A, *S = path.swapped ? A : B;
    const int64_t rows = path.swapped ? N : M, cols = path.swapped ? M : N;
    if (path.kind == StridedPath::kTransposed)
        return gemm_ex<T>(variants, count, path.transa, path.transb, rows, cols, K, alpha, F, path.lda, S, path.ldb, beta, C,
                          path.ldc, stream_, -1);
    hipStream_t stream = (hipStream_t)stream_;
    const int m = (int)M, n = (int)N, k = (int)K;
    (void)hipGetLastError();   // see gemm_ex
    if (!product) {
        if (beta == T(1)) return GEMM_F64_OK;
        return launch_scale<T>(m, n, beta, C, rsc, csc, stream) == hipSuccess ? GEMM_F64_OK : GEMM_F64_ERR_LAUNCH;
    }
    // kSampled: the 64 x 64 tile, the only one the mode is built for
    Job<T> job{path.transa, path.transb, (int)rows, (int)cols, k, alpha, F, path.lda, S, path.ldb, beta, C, path.ldc, stream, 1,
               SplitK{k, 0, 0, 0}};
    job.sampled = true;
    job.es = ElemStrides{path.es_a, path.es_b, path.es_c};
    return launch_mfma<T, 64, 64, 2, 2>(job) == hipSuccess ? GEMM_F64_OK : GEMM_F64_ERR_LAUNCH;
}

}  // namespace gemm_detail
