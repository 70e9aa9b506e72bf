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

#include <type_traits>

namespace gemm_f64_detail {

typedef double v4d __attribute__((ext_vector_type(4)));
typedef double v2d __attribute__((ext_vector_type(2)));

constexpr int kXcds = 8;    // workgroups are dealt round-robin to 8 XCDs, each with a private L2
constexpr int kGroupM = 8;  // tile rows per group of the grouped tile order
constexpr int kBK = 16;     // depth of one LDS stage
constexpr int kThreads = 256;
constexpr int kLean = 0, kGeneric = 1, kStaged = 2;  // kernel modes, see gemm_f64_mfma_kernel

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

// One asynchronous 16-byte-per-lane global->LDS load: lane l copies the 16 bytes at
// sbase + voff(l) to LDS address lds_addr + 16 * l.  Issued as inline asm for two reasons: the
// address is a wave-uniform 64-bit base in SGPRs plus a 32-bit per-lane offset, which costs no
// vector ALU work when the base advances; and the compiler, which answers every LDS dependency
// with a full lgkmcnt(0) drain while it knows such a load to be in flight, does not see it.
// Completion is awaited by the s_waitcnt vmcnt(0) inside stage_barrier().
__device__ __forceinline__ void async_copy16(uint32_t voff, const void *sbase, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(voff), "s"(sbase), "s"(lds_addr)
                 : "memory");
}

// The 4-byte form: lane l copies the 4 bytes at sbase + voff(l) to LDS address lds_addr + 4 * l.
__device__ __forceinline__ void async_copy4(uint32_t voff, const void *sbase, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :
                 : "v"(voff), "s"(sbase), "s"(lds_addr)
                 : "memory");
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
// MODE = kLean: every tile is full, K is a multiple of 16, A and B are 16-byte aligned with even
// leading dimensions (checked on the host); only the asynchronous path is compiled in.
// MODE = kGeneric adds the element-wise, zero-filled path through VGPRs for the ragged last K stage
// (synchronous: once per tile) and handles edge tiles; it also runs unaligned operands (vec_ok = 0)
// through that synchronous path, slowly.
// MODE = kStaged is for unaligned operands: every stage goes through VGPRs, loaded two stages ahead
// and written to LDS one stage ahead, at the price of 16 to 32 more live registers.
template <int BM, int BN, int WM, int WN, int MODE>
__global__ void __launch_bounds__(kThreads, 2)
gemm_f64_mfma_kernel(int M, int N, int K, const double *__restrict__ A, int64_t lda,
                     const double *__restrict__ B, int64_t ldb, double *__restrict__ C, int64_t ldc,
                     int tiles_m, int tiles_n, int vec_ok)
{
    constexpr int BK = kBK;
    constexpr bool GENERIC = MODE != kLean;
    constexpr bool STAGED = MODE == kStaged;
    static_assert(MODE == kLean || MODE == kGeneric || MODE == kStaged, "kernel mode");
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
    // Columns of B to the right of the matrix feed only columns of C that are never stored either;
    // there the lanes whose pair of columns lies outside are switched off (their LDS cells keep
    // stale bits) and, when N is odd, the last column is fetched on its own, four bytes per lane.
    // Only the ragged last K stage goes through VGPRs, for both operands, because there zeros are
    // required: k >= K contributes to every output.
    const int nk_async_a = STAGED ? 0 : GENERIC ? (vec_ok ? K / BK : 0) : nk;
    const int nk_async_b = nk_async_a;
    const bool b_edge = GENERIC && (n0 + BN > N);

    // ---- asynchronous path: each wave issues its share of 1 KiB global->LDS loads -------------
    // A chunk c = (iblk, h): lane l fetches the pair (row iblk*16 + l%16, k pair 4h + l/16).
    // B load r: BN = 128: row r, lane l fetches columns 2l, 2l+1;
    //           BN = 64 : rows 2r and 2r+1, lane l fetches row 2r + l/32, columns 2(l%32), +1.
    // Every address is a wave-uniform 64-bit base, advanced with scalar arithmetic, plus a 32-bit
    // per-lane byte offset computed once: FP64 MFMAs and ordinary vector ALU instructions compete
    // for the same issue cycles on this chip, so the K loop should contain none of the latter.
    // (The host only selects this path when BM * lda * 8 and 2 * ldb * 8 fit in 31 bits.)
    constexpr int A_PER_WAVE = A_CHUNKS / 4, B_PER_WAVE = B_LOADS / 4;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
    uint32_t a_voff[A_PER_WAVE];
#pragma unroll
    for (int q = 0; q < A_PER_WAVE; ++q) {
        const int c = w + 4 * q;
        const int iblk = c >> 1, h = c & 1;
        int row = iblk * 16 + li;
        if (GENERIC) row = (m0 + row < M) ? row : (M - 1 - m0);
        a_voff[q] = (uint32_t)(((int64_t)row * lda + 8 * h + 2 * lg) * 8);
    }
    const uint32_t b_voff =
        (BN == 128) ? (uint32_t)(16 * l) : (uint32_t)((((int64_t)(l >> 5)) * ldb + 2 * (l & 31)) * 8);
    const char *const a_base = reinterpret_cast<const char *>(A + (int64_t)m0 * lda);
    const char *const b_base = reinterpret_cast<const char *>(B + n0);
    auto fetch_async_a = [&](int kt, int buf) {
        const uint32_t dst = lds_base + buf * STAGE + w * 1024;
        const char *src = a_base + (int64_t)kt * (BK * 8);
#pragma unroll
        for (int q = 0; q < A_PER_WAVE; ++q) async_copy16(a_voff[q], src, dst + q * 4096);
    };
    auto fetch_async_b = [&](int kt, int buf) {
        // r = w + 4q: destination (r / 2) * B_PAIR + (r % 2) * B_ROW for BN = 128, r * B_PAIR for BN = 64
        const uint32_t dst = lds_base + buf * STAGE + A_STAGE +
                             ((BN == 128) ? (w >> 1) * B_PAIR + (w & 1) * B_ROW : w * B_PAIR);
        const int64_t row_bytes = ldb * 8;
        const char *src = b_base + (int64_t)(kt * BK + (BN == 128 ? w : 2 * w)) * row_bytes;
        if (!b_edge) {
#pragma unroll
            for (int q = 0; q < B_PER_WAVE; ++q)
                async_copy16(b_voff, src + (int64_t)(BN == 128 ? 4 * q : 8 * q) * row_bytes,
                             dst + q * ((BN == 128) ? 2 * B_PAIR : 4 * B_PAIR));
        } else {
            const int valid = N - n0;                     // 1 .. BN-1 columns of this tile exist
            const bool pair_ok = 2 * (l % JP) + 1 < valid;
            const int jt = valid - 1;                     // last column; fetched alone when valid is odd
#pragma unroll
            for (int q = 0; q < B_PER_WAVE; ++q) {
                const char *rsrc = src + (int64_t)(BN == 128 ? 4 * q : 8 * q) * row_bytes;
                const uint32_t rdst = dst + q * ((BN == 128) ? 2 * B_PAIR : 4 * B_PAIR);
                if (pair_ok) async_copy16(b_voff, rsrc, rdst);
                if ((valid & 1) && l < 2) {
                    async_copy4(4 * l, rsrc + jt * 8, rdst + jt * 8);
                    if (BN == 64) async_copy4(4 * l, rsrc + row_bytes + jt * 8, rdst + B_ROW + jt * 8);
                }
            }
        }
    };

    // ---- VGPR path (right-edge tiles, ragged K, unaligned operands): element-wise loads, zero
    // outside the logical matrices, written to LDS in the same layout.  Both operands are zeroed
    // for k >= K, so padding only ever forms 0 * 0.  Synchronous: used where it is rare.
    auto load_regs_a = [&](int kt, double (&ra)[2 * NA]) {
        const int k0 = kt * BK;
#pragma unroll
        for (int q = 0; q < NA; ++q) {
            const int row = m0 + li + 16 * w + 64 * (q >> 1), k = k0 + 2 * (lg + 4 * (q & 1));
            const double *p = A + (int64_t)row * lda + k;
            ra[2 * q] = (row < M && k < K) ? p[0] : 0.0;
            ra[2 * q + 1] = (row < M && k + 1 < K) ? p[1] : 0.0;
        }
    };
    auto store_regs_a = [&](int buf, const double (&ra)[2 * NA]) {
        char *stage = lds + buf * STAGE;
#pragma unroll
        for (int q = 0; q < NA; ++q) {
            const int i = li + 16 * w + 64 * (q >> 1), kp = lg + 4 * (q & 1);
            v2d v;
            v.x = ra[2 * q];
            v.y = ra[2 * q + 1];
            *reinterpret_cast<v2d *>(stage + (((i >> 4) << 1) | (kp >> 2)) * 1024 + (kp & 3) * 256 + (i & 15) * 16) = v;
        }
    };
    auto load_regs_b = [&](int kt, double (&rb)[2 * NB]) {
        const int k0 = kt * BK;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int kk = k0 + l / JP + (64 / JP) * w + (kThreads / JP) * q, col = n0 + 2 * (l % JP);
            const double *p = B + (int64_t)kk * ldb + col;
            rb[2 * q] = (kk < K && col < N) ? p[0] : 0.0;
            rb[2 * q + 1] = (kk < K && col + 1 < N) ? p[1] : 0.0;
        }
    };
    auto store_regs_b = [&](int buf, const double (&rb)[2 * NB]) {
        char *stage = lds + buf * STAGE;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int kk = l / JP + (64 / JP) * w + (kThreads / JP) * q, j = 2 * (l % JP);
            v2d v;
            v.x = rb[2 * q];
            v.y = rb[2 * q + 1];
            *reinterpret_cast<v2d *>(stage + A_STAGE + (kk >> 1) * B_PAIR + (kk & 1) * B_ROW + j * 8) = v;
        }
    };
    auto fetch_sync_a = [&](int kt, int buf) {
        double ra[2 * NA];
        load_regs_a(kt, ra);
        store_regs_a(buf, ra);
    };
    auto fetch_sync_b = [&](int kt, int buf) {
        double rb[2 * NB];
        load_regs_b(kt, rb);
        store_regs_b(buf, rb);
    };
    // kStaged: the registers that carry a stage from its loads (after one barrier) to its LDS
    // writes (before the next)
    double sa[STAGED ? 2 * NA : 1], sb[STAGED ? 2 * NB : 1];
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
    (void)sa;
    (void)sb;

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

    // MFMAs lo .. hi-1 of the 2 * MI * NI that consume one half-stage, in the order e, mi, ni
    auto mfma_range = [&](const v2d (&fa)[MI], const v2d (&fb)[NI], int lo, int hi) {
#pragma unroll
        for (int idx = 0; idx < 2 * MI * NI; ++idx) {
            if (idx < lo || idx >= hi) continue;
            const int e = idx / (MI * NI), mi = (idx / NI) % MI, ni = idx % NI;
            acc[mi][ni] = __builtin_amdgcn_mfma_f64_16x16x4f64(e ? fa[mi].y : fa[mi].x, e ? fb[ni].y : fb[ni].x,
                                                               acc[mi][ni], 0, 0, 0);
        }
    };
    constexpr int HALF = 2 * MI * NI;

    v2d fa0[MI], fb0[NI], fa1[MI], fb1[NI];

    // prologue: stages 0 and 1
    for (int kt = 0; kt < 2 && kt < nk; ++kt) {
        fetch_early(kt, kt);
        fetch_late(kt, kt);
    }
    stage_barrier();
    read_frags(0, 0, fa0, fb0);

    // Stage s lives in buffer s % 2.  Per iteration: the second half's fragments are read while the
    // first half's MFMAs run; then one barrier, after which buffer s % 2 is free for stage s + 2 and
    // stage s + 1 (fetched one iteration ago) is complete, so its first fragments are read and the
    // next fetch is issued underneath the second half's MFMAs.  The loop is unrolled by two so that
    // the buffer index is a compile-time constant and every LDS address is base register + immediate.
    auto iteration = [&](int s, auto cur_tag) {
        constexpr int cur = decltype(cur_tag)::value;
        // The first MFMAs wait for fragments that were requested long ago; only then are the next
        // reads queued, so that wait never covers a read that has just been issued.
        mfma_range(fa0, fb0, 0, NI);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(cur, 1, fa1, fb1);
        __builtin_amdgcn_sched_barrier(0);
        mfma_range(fa0, fb0, NI, HALF);
        if constexpr (STAGED) {
            if (s >= 1 && s + 1 < nk) {  // stage s + 1 was loaded during the previous iteration
                store_regs_a(cur ^ 1, reinterpret_cast<const double(&)[2 * NA]>(sa));
                store_regs_b(cur ^ 1, reinterpret_cast<const double(&)[2 * NB]>(sb));
            }
        } else if (GENERIC && s >= 1 && s + 1 < nk) {
            fetch_late(s + 1, cur ^ 1);
        }
        stage_barrier();
        // unconditional (in the last iteration it re-reads a stale buffer and the values are never
        // used): the number of LDS reads in flight is then the same on every path, and the compiler
        // waits for exactly the older ones before the MFMAs below instead of draining the queue
        read_frags(cur ^ 1, 0, fa0, fb0);
        if constexpr (STAGED) {
            if (s + 2 < nk) {
                load_regs_a(s + 2, reinterpret_cast<double(&)[2 * NA]>(sa));
                load_regs_b(s + 2, reinterpret_cast<double(&)[2 * NB]>(sb));
            }
        } else if (s + 2 < nk) {
            fetch_early(s + 2, cur);
        }
        __builtin_amdgcn_sched_barrier(0);
        mfma_range(fa1, fb1, 0, HALF);
    };
    int s = 0;
    for (; s + 1 < nk; s += 2) {
        iteration(s, std::integral_constant<int, 0>{});
        iteration(s + 1, std::integral_constant<int, 1>{});
    }
    if (s < nk) iteration(s, std::integral_constant<int, 0>{});

    // C is read and written exactly once per element, after the K loop.  Loads are issued in batches
    // of two 16-row blocks (up to 32 per lane in flight) before the first is consumed: the epilogue
    // is latency-bound, so its duration is the number of batches times the memory latency.
    const int row_base = m0 + wm * TM + lg;
    const int col_base = n0 + wn * TN + li;
    constexpr int MB = (MI >= 2) ? 2 : 1;
#pragma unroll
    for (int mb = 0; mb < MI; mb += MB) {
        double cin[MB][NI][4];
#pragma unroll
        for (int mi = mb; mi < mb + MB; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = row_base + mi * 16 + 4 * r, col = col_base + ni * 16;
                    if (!GENERIC || tile_full || (row < M && col < N)) cin[mi - mb][ni][r] = C[(int64_t)row * ldc + col];
                    else cin[mi - mb][ni][r] = 0.0;
                }
#pragma unroll
        for (int mi = mb; mi < mb + MB; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = row_base + mi * 16 + 4 * r, col = col_base + ni * 16;
                    if (!GENERIC || tile_full || (row < M && col < N))
                        C[(int64_t)row * ldc + col] = cin[mi - mb][ni][r] + acc[mi][ni][r];
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
