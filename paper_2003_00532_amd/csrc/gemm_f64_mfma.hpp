// FP64 MFMA GEMM kernels for gfx950 (MI355X): C += A * B, row-major.
//
// How the paper's scheme maps onto this kernel (Section 2.4 schedule, Sections
// 2.6, 2.7, 2.9, 2.10, 2.14):
//   * cache tile (M_C x K_C block of A, K_C x N_R panel of B)  ->  workgroup macro-tile BM x BN with a
//     BK-deep slice of A and B staged in LDS ("packing" into a contiguous, conflict-free layout);
//   * register tile M_R x N_R, unroll-and-jammed and scalar-replaced  ->  per-wave grid of
//     16x16 accumulator tiles of v_mfma_f64_16x16x4_f64 that stay in VGPRs for the whole K loop,
//     C touched exactly once per element;
//   * K_U unrolling  ->  the BK/4 MFMA k-steps of one LDS stage, fully unrolled;
//   * the packed-buffer layout map (i floordiv M_R, k, i mod M_R)  ->  the LDS layout below, chosen
//     so that an MFMA operand fetch is one contiguous, conflict-free LDS read per wave;
//   * the prefetching the paper found missing  ->  slices are fetched one full stage ahead by
//     asynchronous global->LDS loads (no register staging), LDS is double-buffered along K, and
//     operand fragments are read one half-stage ahead of the MFMAs that consume them.
//
// Lane layout of v_mfma_f64_16x16x4_f64 on gfx950, measured with one-hot operands (the test-suite
// re-checks it on the device): with lane l in 0..63,
//   A operand: one double, element (i = l % 16, k = l / 16)
//   B operand: one double, element (k = l / 16, j = l % 16)
//   D / C:     four doubles, register r holds element (i = 4 * r + l / 16, j = l % 16).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gemm_f64_detail {

typedef double v4d __attribute__((ext_vector_type(4)));
typedef double v2d __attribute__((ext_vector_type(2)));

constexpr int kXcds = 8;    // workgroups are dealt round-robin to 8 XCDs, each with a private L2
constexpr int kGroupM = 8;  // tile rows per group of the grouped tile order
constexpr int kBK = 16;     // depth of one LDS stage
constexpr int kThreads = 256;

// Workgroup id -> tile coordinates.  Block b runs on XCD b % kXcds.  Each XCD receives a
// contiguous run of the "grouped" tile order (kGroupM tile rows at a time, column by column
// inside a group), so the ~2 * CUs-per-XCD workgroups resident on one XCD at any moment form a
// compact patch of C and re-use each other's A and B panels in that XCD's L2.
__host__ __device__ inline void tile_of_block(int64_t b, int64_t tiles_m, int64_t tiles_n,
                                              int64_t &tm, int64_t &tn)
{
    const int64_t total = tiles_m * tiles_n;
    const int64_t per = total / kXcds, rem = total % kXcds;
    const int64_t x = b % kXcds, s = b / kXcds;
    const int64_t start = x * per + (x < rem ? x : rem);
    const int64_t logical = start + s;
    const int64_t width = kGroupM * tiles_n;
    const int64_t g = logical / width;
    const int64_t first_m = g * kGroupM;
    const int64_t gsz = (tiles_m - first_m) < kGroupM ? (tiles_m - first_m) : kGroupM;
    const int64_t in_g = logical % width;
    tm = first_m + in_g % gsz;
    tn = in_g / gsz;
}

typedef const __attribute__((address_space(1))) void *global_cptr;
typedef __attribute__((address_space(3))) void *lds_ptr;

// Workgroup barrier that also publishes this wave's LDS traffic: every LDS read, LDS write and
// asynchronous global->LDS load the wave has issued is complete before it arrives.  Written as one
// volatile asm statement with a memory clobber so that the compiler keeps every memory access on
// the side of the barrier where the source puts it (with the barrier builtin and fences, LDS reads
// were observed to sink below the barrier, into the window where other waves refill the buffer).
__device__ __forceinline__ void stage_barrier()
{
    __builtin_amdgcn_sched_barrier(0);  // nothing, MFMAs included, is scheduled across
    asm volatile("s_waitcnt vmcnt(0) expcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// The compiler cannot see an s_waitcnt inside an asm statement, and while an asynchronous
// global->LDS load is in flight it answers every LDS dependency with a full lgkmcnt(0) drain, which
// would expose the latency of the youngest fragment reads.  So the waits are placed by hand, at
// points where only old reads are outstanding, and the fragment registers are passed through the
// asm as read-write operands: afterwards the compiler regards them as complete.
//   BARRIER = true : wait for everything (LDS reads and writes, global->LDS loads), then s_barrier;
//   BARRIER = false: wait for outstanding LDS reads only.
template <bool BARRIER, int NA_, int NB_>
__device__ __forceinline__ void settle(v2d (&fa)[NA_], v2d (&fb)[NB_])
{
    static_assert((NA_ == 2 || NA_ == 4) && (NB_ == 2 || NB_ == 4), "two or four fragments per operand");
    __builtin_amdgcn_sched_barrier(0);  // nothing, MFMAs included, is scheduled across
#define GEMM_F64_SETTLE(...)                                                                              \
    do {                                                                                                  \
        if (BARRIER)                                                                                      \
            asm volatile("s_waitcnt vmcnt(0) expcnt(0) lgkmcnt(0)\n\ts_barrier" : __VA_ARGS__::"memory"); \
        else                                                                                              \
            asm volatile("s_waitcnt lgkmcnt(0)" : __VA_ARGS__::"memory");                                 \
    } while (0)
    if (NA_ == 4 && NB_ == 4)
        GEMM_F64_SETTLE("+v"(fa[0]), "+v"(fa[1]), "+v"(fa[NA_ - 2]), "+v"(fa[NA_ - 1]), "+v"(fb[0]), "+v"(fb[1]),
                        "+v"(fb[NB_ - 2]), "+v"(fb[NB_ - 1]));
    else if (NA_ == 4)
        GEMM_F64_SETTLE("+v"(fa[0]), "+v"(fa[1]), "+v"(fa[NA_ - 2]), "+v"(fa[NA_ - 1]), "+v"(fb[0]), "+v"(fb[1]));
    else if (NB_ == 4)
        GEMM_F64_SETTLE("+v"(fa[0]), "+v"(fa[1]), "+v"(fb[0]), "+v"(fb[1]), "+v"(fb[NB_ - 2]), "+v"(fb[NB_ - 1]));
    else
        GEMM_F64_SETTLE("+v"(fa[0]), "+v"(fa[1]), "+v"(fb[0]), "+v"(fb[1]));
#undef GEMM_F64_SETTLE
    __builtin_amdgcn_sched_barrier(0);
}

// One workgroup = 256 threads = 4 waves arranged WM x WN; each wave owns a (BM/WM) x (BN/WN)
// patch of the macro-tile as MI x NI accumulator tiles of 16 x 16.
//
// LDS layout of one stage (BK = 16 values of k), chosen so that every access is contiguous:
//   A: 1 KiB chunks indexed [i / 16][h], h = (k / 2) / 4; inside a chunk the 16-byte cell of
//      lane-slot (kq, ii), kq = (k / 2) % 4, ii = i % 16, sits at (kq * 16 + ii) * 16 and holds
//      the pair (A[i][2*(4h+kq)], A[i][2*(4h+kq)+1]).  A wave's MFMA operand fetch for one 16-row
//      block and one h is then a single 1 KiB lane-linear ds_read_b128, and its two halves feed
//      two MFMA k-steps: step e uses k = 2*(4h + l/16) + e in lane group l/16.
//   B: row pairs [k / 2] at a stride of 2*BN*8 + 128 bytes, the two rows of a pair BN*8 apart; a
//      lane reads B[2*(4h + l/16) + e][j] for e = 0, 1 with one ds_read2_b64.  The pair stride is
//      128 mod 256 bytes, so the two 16-lane groups served together fall in different bank halves.
// Both layouts are exactly what a 16-byte-per-lane global->LDS load writes (lane-linear 1 KiB), so
// full tiles are staged with global_load_lds_dwordx4 and never pass through VGPRs.
//
// GENERIC = false: every tile is full, K is a multiple of 16, A and B are 16-byte aligned with
// even leading dimensions (checked on the host).  GENERIC = true adds the element-wise, zero-filled
// path through VGPRs for edge tiles, the ragged last K stage and unaligned operands (vec_ok = 0).
template <int BM, int BN, int WM, int WN, bool GENERIC>
__global__ void __launch_bounds__(kThreads, 2)
gemm_f64_mfma_kernel(int M, int N, int K, const double *__restrict__ A, int64_t lda,
                     const double *__restrict__ B, int64_t ldb, double *__restrict__ C, int64_t ldc,
                     int tiles_m, int tiles_n, int vec_ok)
{
    constexpr int BK = kBK;
    static_assert(WM * WN == 4, "four waves per workgroup");
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int MI = TM / 16, NI = TN / 16;
    static_assert(MI >= 1 && NI >= 1 && TM % 16 == 0 && TN % 16 == 0, "wave tile is a grid of 16x16 tiles");
    static_assert(BM % 64 == 0 && (BN == 64 || BN == 128), "supported macro-tiles");
    constexpr int A_CHUNKS = (BM / 16) * 2;
    constexpr int A_STAGE = A_CHUNKS * 1024;          // bytes
    constexpr int B_ROW = BN * 8;                     // bytes between the two rows of a k pair
    constexpr int B_PAIR = 2 * B_ROW + 128;           // bytes between k pairs
    static_assert(B_PAIR % 256 == 128, "pair stride must be 128 mod 256 bytes");
    constexpr int B_STAGE = (BK / 2) * B_PAIR;
    constexpr int STAGE = A_STAGE + B_STAGE;
    constexpr int B_LOADS = (BK * BN * 8) / 1024;     // 1 KiB global->LDS loads per B stage
    constexpr int NA = BM / 32, NB = BN / 32;         // 16-byte pairs per thread per stage (VGPR path)
    constexpr int JP = BN / 2;

    __shared__ __attribute__((aligned(1024))) char lds[2 * STAGE];

    const int t = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int l = t & 63;
    const int wm = w / WN, wn = w % WN;
    const int lg = l >> 4, li = l & 15;

    int64_t tm64, tn64;
    tile_of_block(blockIdx.x, tiles_m, tiles_n, tm64, tn64);
    const int m0 = (int)tm64 * BM, n0 = (int)tn64 * BN;

    const bool tile_full = (m0 + BM <= M) && (n0 + BN <= N);
    const int nk = (K + BK - 1) / BK;
    // Number of leading stages fetched by the asynchronous global->LDS path, per operand.  Rows of
    // an A tile that lie below the matrix are redirected to row M - 1: they only feed rows of C
    // that are never stored, so no zero fill is needed in M and such tiles stay on the fast path.
    // Columns of B to the right of the matrix cannot be redirected pairwise (N may be odd), so
    // tiles on the right edge stage B through VGPRs.  The ragged last K stage always does, for
    // both operands, because there zeros are required.
    const int nk_async_a = GENERIC ? (vec_ok ? K / BK : 0) : nk;
    const int nk_async_b = GENERIC ? ((vec_ok && n0 + BN <= N) ? K / BK : 0) : nk;

    // ---- asynchronous path: each wave issues its share of 1 KiB global->LDS loads -------------
    // A chunk c = (iblk, h): lane l fetches the pair (row iblk*16 + l%16, k pair 4h + l/16).
    // B load r: BN = 128: row r, lane l fetches columns 2l, 2l+1;
    //           BN = 64 : rows 2r and 2r+1, lane l fetches row 2r + l/32, columns 2(l%32), +1.
    const double *b_src = (BN == 128) ? B + (int64_t)(n0 + 2 * l)
                                      : B + (int64_t)(l >> 5) * ldb + (n0 + 2 * (l & 31));
    auto fetch_async_a = [&](int kt, int buf) {
        char *stage = lds + buf * STAGE;
        const int k0 = kt * BK;
#pragma unroll
        for (int q = 0; q < A_CHUNKS / 4; ++q) {
            const int c = w + 4 * q;
            const int iblk = c >> 1, h = c & 1;
            int row = m0 + iblk * 16 + li;
            if (GENERIC) row = row < M ? row : M - 1;
            __builtin_amdgcn_global_load_lds((global_cptr)(A + (int64_t)row * lda + (k0 + 8 * h + 2 * lg)),
                                             (lds_ptr)(stage + c * 1024), 16, 0, 0);
        }
    };
    auto fetch_async_b = [&](int kt, int buf) {
        char *stage = lds + buf * STAGE;
        const int k0 = kt * BK;
#pragma unroll
        for (int q = 0; q < B_LOADS / 4; ++q) {
            const int r = w + 4 * q;
            if (BN == 128)
                __builtin_amdgcn_global_load_lds((global_cptr)(b_src + (int64_t)(k0 + r) * ldb),
                                                 (lds_ptr)(stage + A_STAGE + (r >> 1) * B_PAIR + (r & 1) * B_ROW), 16, 0, 0);
            else
                __builtin_amdgcn_global_load_lds((global_cptr)(b_src + (int64_t)(k0 + 2 * r) * ldb),
                                                 (lds_ptr)(stage + A_STAGE + r * B_PAIR), 16, 0, 0);
        }
    };

    // ---- VGPR path (right-edge tiles, ragged K, unaligned operands): element-wise loads, zero
    // outside the logical matrices, written to LDS in the same layout.  Both operands are zeroed
    // for k >= K, so padding only ever forms 0 * 0.  Synchronous: used where it is rare.
    auto fetch_sync_a = [&](int kt, int buf) {
        char *stage = lds + buf * STAGE;
        const int k0 = kt * BK;
        double ra[2 * NA];
#pragma unroll
        for (int q = 0; q < NA; ++q) {
            const int row = m0 + li + 16 * w + 64 * (q >> 1), k = k0 + 2 * (lg + 4 * (q & 1));
            const double *p = A + (int64_t)row * lda + k;
            ra[2 * q] = (row < M && k < K) ? p[0] : 0.0;
            ra[2 * q + 1] = (row < M && k + 1 < K) ? p[1] : 0.0;
        }
#pragma unroll
        for (int q = 0; q < NA; ++q) {
            const int i = li + 16 * w + 64 * (q >> 1), kp = lg + 4 * (q & 1);
            v2d v;
            v.x = ra[2 * q];
            v.y = ra[2 * q + 1];
            *reinterpret_cast<v2d *>(stage + (((i >> 4) << 1) | (kp >> 2)) * 1024 + (kp & 3) * 256 + (i & 15) * 16) = v;
        }
    };
    auto fetch_sync_b = [&](int kt, int buf) {
        char *stage = lds + buf * STAGE;
        const int k0 = kt * BK;
        double rb[2 * NB];
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int kk = k0 + l / JP + (64 / JP) * w + (kThreads / JP) * q, col = n0 + 2 * (l % JP);
            const double *p = B + (int64_t)kk * ldb + col;
            rb[2 * q] = (kk < K && col < N) ? p[0] : 0.0;
            rb[2 * q + 1] = (kk < K && col + 1 < N) ? p[1] : 0.0;
        }
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int kk = l / JP + (64 / JP) * w + (kThreads / JP) * q, j = 2 * (l % JP);
            v2d v;
            v.x = rb[2 * q];
            v.y = rb[2 * q + 1];
            *reinterpret_cast<v2d *>(stage + A_STAGE + (kk >> 1) * B_PAIR + (kk & 1) * B_ROW + j * 8) = v;
        }
    };
    // issue what can be fetched asynchronously for stage kt (as early as its buffer is free) ...
    auto fetch_early = [&](int kt, int buf) {
        if (kt < nk_async_a) fetch_async_a(kt, buf);
        if (kt < nk_async_b) fetch_async_b(kt, buf);
    };
    // ... and fetch the rest synchronously just before the barrier that publishes the stage
    auto fetch_late = [&](int kt, int buf) {
        if (!GENERIC) return;
        if (kt >= nk_async_a) fetch_sync_a(kt, buf);
        if (kt >= nk_async_b) fetch_sync_b(kt, buf);
    };

    // ---- operand fragments: one half-stage (h) = two MFMA k-steps ------------------------------
    const int a_frag = ((wm * (TM / 16)) << 1) * 1024 + l * 16;              // + mi*2048 + h*1024
    const int b_frag = A_STAGE + lg * B_PAIR + (wn * TN + li) * 8;           // + h*4*B_PAIR + ni*128
    auto read_frags = [&](int buf, int h, v2d (&fa)[MI], v2d (&fb)[NI]) {
        const char *stage = lds + buf * STAGE;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
            fa[mi] = *reinterpret_cast<const v2d *>(stage + a_frag + mi * 2048 + h * 1024);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const char *p = stage + b_frag + h * 4 * B_PAIR + ni * 128;
            fb[ni].x = *reinterpret_cast<const double *>(p);
            fb[ni].y = *reinterpret_cast<const double *>(p + B_ROW);
        }
    };

    v4d acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = v4d{0.0, 0.0, 0.0, 0.0};

    auto mfma_half = [&](const v2d (&fa)[MI], const v2d (&fb)[NI]) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                acc[mi][ni] = __builtin_amdgcn_mfma_f64_16x16x4f64(fa[mi].x, fb[ni].x, acc[mi][ni], 0, 0, 0);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                acc[mi][ni] = __builtin_amdgcn_mfma_f64_16x16x4f64(fa[mi].y, fb[ni].y, acc[mi][ni], 0, 0, 0);
    };

    v2d fa0[MI], fb0[NI], fa1[MI], fb1[NI];

    // prologue: stages 0 and 1
    for (int kt = 0; kt < 2 && kt < nk; ++kt) {
        fetch_early(kt, kt);
        fetch_late(kt, kt);
    }
    stage_barrier();
    read_frags(0, 0, fa0, fb0);
    settle<false>(fa0, fb0);

    // Stage s lives in buffer s % 2.  Per iteration: the second half's fragments are read while the
    // first half's MFMAs run; then one barrier, after which buffer s % 2 is free for stage s + 2 and
    // stage s + 1 (fetched one iteration ago) is complete, so its first fragments are read and the
    // next fetch is issued underneath the second half's MFMAs.
    for (int s = 0; s < nk; ++s) {
        const int cur = s & 1;
        read_frags(cur, 1, fa1, fb1);
        __builtin_amdgcn_sched_barrier(0);  // issue the reads first, then the MFMAs that hide them
        mfma_half(fa0, fb0);
        if (s >= 1 && s + 1 < nk) fetch_late(s + 1, cur ^ 1);
        settle<true>(fa1, fb1);
        // unconditional (in the last iteration it re-reads a stale buffer and the values are never
        // used): a fixed number of LDS reads in flight lets the compiler wait for exactly the older
        // ones before the MFMAs below instead of draining the queue
        read_frags(cur ^ 1, 0, fa0, fb0);
        if (s + 2 < nk) fetch_early(s + 2, cur);
        mfma_half(fa1, fb1);
        settle<false>(fa0, fb0);  // the reads issued 32 MFMAs ago have long landed
    }

    // C is read and written exactly once per element, after the K loop.
    const int row_base = m0 + wm * TM + lg;
    const int col_base = n0 + wn * TN + li;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        double cin[NI][4];
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = row_base + mi * 16 + 4 * r, col = col_base + ni * 16;
                if (!GENERIC || tile_full || (row < M && col < N)) cin[ni][r] = C[(int64_t)row * ldc + col];
                else cin[ni][r] = 0.0;
            }
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = row_base + mi * 16 + 4 * r, col = col_base + ni * 16;
                if (!GENERIC || tile_full || (row < M && col < N))
                    C[(int64_t)row * ldc + col] = cin[ni][r] + acc[mi][ni][r];
            }
    }
}

// Reference-shaped kernel without tiling or staging: one thread per element of C, k ascending.
// Kept as the bottom rung of the ladder (the paper's Section 2.3 starting point) and as an
// on-device cross-check that shares nothing with the MFMA kernel.
__global__ void __launch_bounds__(256)
gemm_f64_naive_kernel(int M, int N, int K, const double *__restrict__ A, int64_t lda,
                      const double *__restrict__ B, int64_t ldb, double *__restrict__ C, int64_t ldc)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)M * N) return;
    const int i = (int)(idx / N), j = (int)(idx % N);
    double c = C[(int64_t)i * ldc + j];
    const double *a = A + (int64_t)i * lda;
    for (int k = 0; k < K; ++k) c += a[k] * B[(int64_t)k * ldb + j];
    C[(int64_t)i * ldc + j] = c;
}

}  // namespace gemm_f64_detail
