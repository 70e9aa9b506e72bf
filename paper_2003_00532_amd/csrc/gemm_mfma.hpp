// MFMA GEMM kernels for gfx950 (MI355X): C += A * B, row-major, for double and float elements.
//
// How the paper's scheme maps onto this kernel (Section 2.4 schedule, Sections
// 2.6, 2.7, 2.9, 2.10, 2.13, 2.14):
//   * cache tile (M_C x K_C block of A, K_C x N_R panel of B)  ->  workgroup macro-tile BM x BN with a
//     BK-deep slice of A and B staged in LDS ("packing" into a contiguous, conflict-free layout);
//   * register tile M_R x N_R, unroll-and-jammed and scalar-replaced  ->  per-wave grid of
//     16x16 accumulator tiles of a 16x16x4 MFMA that stay in VGPRs for the whole K loop,
//     C touched exactly once per element;
//   * K_U unrolling  ->  the BK/4 MFMA k-steps of one LDS stage, fully unrolled;
//   * the packed-buffer layout map (i floordiv M_R, k, i mod M_R)  ->  the LDS layout below, chosen
//     so that an MFMA operand fetch is one contiguous, conflict-free LDS read per wave;
//   * the prefetching the paper found missing  ->  slices are fetched one full stage ahead by
//     asynchronous global->LDS loads (no register staging), LDS is double-buffered along K, and
//     operand fragments are read one half-stage ahead of the MFMAs that consume them;
//   * SGEMM by substituting the element type and doubling the elements per vector  ->  the same
//     kernel with four floats instead of two doubles per 16-byte cell and a stage twice as deep.
//
// Lane layouts on gfx950, measured with one-hot operands (the test-suite re-checks them on the
// device): with lane l in 0..63, both v_mfma_f64_16x16x4_f64 and v_mfma_f32_16x16x4_f32 take
//   A operand: one element, (i = l % 16, k = l / 16)
//   B operand: one element, (k = l / 16, j = l % 16)
// and return four elements per lane, register r holding
//   f64: (i = 4 * r + l / 16, j = l % 16)          f32: (i = 4 * (l / 16) + r, j = l % 16).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace gemm_detail {

typedef double v4d __attribute__((ext_vector_type(4)));
typedef double v2d __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kXcds = 8;    // workgroups are dealt round-robin to 8 XCDs, each with a private L2
constexpr int kGroupM = 8;  // tile rows per group of the grouped tile order
constexpr int kThreads = 256;
constexpr int kLean = 0, kGeneric = 1, kStaged = 2;  // kernel modes, see gemm_mfma_kernel

// What depends on the element type.  A 16-byte LDS cell holds E consecutive k (for A) of one row;
// one LDS stage is 8 cells deep, so BK = 8 * E (16 for double, 32 for float).
template <typename T> struct Elem;
template <> struct Elem<double> {
    static constexpr int E = 2;
    typedef v2d cell_t;
    typedef v4d acc_t;
    static __device__ __forceinline__ acc_t mfma(double a, double b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int d_row(int r, int lg) { return 4 * r + lg; }
};
template <> struct Elem<float> {
    static constexpr int E = 4;
    typedef v4f cell_t;
    typedef v4f acc_t;
    static __device__ __forceinline__ acc_t mfma(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int d_row(int r, int lg) { return 4 * lg + r; }
};

// Workgroup id -> tile coordinates.  Block b runs on XCD b % kXcds.  Each XCD receives a
// contiguous run of the "grouped" tile order (kGroupM tile rows at a time, column by column
// inside a group), so the workgroups resident on one XCD at any moment form a compact patch of C
// and re-use each other's A and B panels in that XCD's L2.
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
// LDS layout of one stage (BK = 8 * E values of k), chosen so that every access is contiguous:
//   A: 1 KiB chunks indexed [i / 16][h], h = kc / 4 with kc = k / E the cell index along k; inside a
//      chunk the 16-byte cell of lane-slot (kq, ii), kq = kc % 4, ii = i % 16, sits at
//      (kq * 16 + ii) * 16 and holds A[i][E*kc .. E*kc + E-1].  A wave's MFMA operand fetch for one
//      16-row block and one h is then a single 1 KiB lane-linear ds_read_b128, and its E elements
//      feed E MFMA k-steps: step e uses k = E * (4h + l/16) + e in lane group l/16.
//   B: groups of E rows [k / E] at a stride of E*BN*sizeof(T) + 16*sizeof(T) bytes, the rows of a
//      group BN*sizeof(T) apart; a lane reads B[E*(4h + l/16) + e][j] for e = 0..E-1.  The group
//      stride is 16*sizeof(T) modulo 256 bytes, so the 16-lane groups that are served together
//      fall into different banks.
// Both layouts are exactly what a 16-byte-per-lane global->LDS load writes (lane-linear 1 KiB), so
// full tiles are staged with global_load_lds_dwordx4 and never pass through VGPRs.
//
// MODE = kLean: every tile is full, K is a multiple of BK, A and B are 16-byte aligned with
// leading dimensions that are multiples of E (checked on the host); only the asynchronous path is
// compiled in.
// MODE = kGeneric adds the element-wise, zero-filled path through VGPRs for the ragged last K stage
// (synchronous: once per tile) and handles edge tiles.
// MODE = kStaged is for unaligned operands: every stage goes through VGPRs, loaded two stages ahead
// and written to LDS one stage ahead, at the price of 16 to 32 more live registers.
template <typename T, int BM, int BN, int WM, int WN, int MODE>
__global__ void __launch_bounds__(kThreads, 2)
gemm_mfma_kernel(int M, int N, int K, const T *__restrict__ A, int64_t lda, const T *__restrict__ B, int64_t ldb,
                 T *__restrict__ C, int64_t ldc, int tiles_m, int tiles_n)
{
    typedef Elem<T> EL;
    typedef typename EL::cell_t cell_t;
    typedef typename EL::acc_t acc_t;
    constexpr int E = EL::E;
    constexpr int SZ = (int)sizeof(T);
    static_assert(E * SZ == 16, "a cell is 16 bytes");
    constexpr int BK = 8 * E;
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
    constexpr int B_ROW = BN * SZ;                    // bytes between consecutive k rows of a group
    constexpr int B_GROUP = E * B_ROW + 16 * SZ;      // bytes between groups of E rows
    static_assert(B_GROUP % 256 == 16 * SZ, "group stride must be 16 elements modulo 256 bytes");
    constexpr int B_STAGE = 8 * B_GROUP;
    constexpr int STAGE = A_STAGE + B_STAGE;
    constexpr int B_LOADS = (BK * BN * SZ) / 1024;    // 1 KiB global->LDS loads per B stage
    constexpr int RPI = 1024 / B_ROW;                 // B rows covered by one such load
    constexpr int LPR = 64 / RPI;                     // lanes per row in it
    static_assert(RPI >= 1 && RPI <= E && E % RPI == 0, "a load stays inside one group of rows");
    constexpr int NA = BM / 32, NB = BN / 32;         // 16-byte cells per thread per stage (VGPR path)
    constexpr int CPR = BN / E;                       // cells per B row
    static_assert(64 % CPR == 0, "a wave covers whole B rows of cells");

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
    // Number of leading stages fetched by the asynchronous global->LDS path.  Rows of an A tile that
    // lie below the matrix are redirected to row M - 1: they only feed rows of C that are never
    // stored, so no zero fill is needed in M and such tiles stay on the fast path.  Columns of B to
    // the right of the matrix feed only columns of C that are never stored either; there the lanes
    // whose cell of columns lies outside are switched off (their LDS cells keep stale bits) and a
    // partly valid last cell is fetched on its own, four bytes per lane.  Only the ragged last K
    // stage goes through VGPRs, for both operands, because there zeros are required: k >= K
    // contributes to every output.
    const int nk_async = STAGED ? 0 : GENERIC ? K / BK : nk;
    const bool b_edge = GENERIC && (n0 + BN > N);

    // ---- asynchronous path: each wave issues its share of 1 KiB global->LDS loads -------------
    // A chunk c = (iblk, h): lane l fetches the cell (row iblk*16 + l%16, cell 4h + l/16 along k).
    // B load r covers rows r*RPI .. r*RPI + RPI-1: lane l fetches row r*RPI + l/LPR, cell l%LPR.
    // Every address is a wave-uniform 64-bit base, advanced with scalar arithmetic, plus a 32-bit
    // per-lane byte offset computed once: MFMAs and ordinary vector ALU instructions compete for
    // the same issue cycles on this chip, so the K loop should contain none of the latter.
    // (The host only selects this path when BM * lda and E * ldb, in bytes, fit in 31 bits.)
    constexpr int A_PER_WAVE = A_CHUNKS / 4, B_PER_WAVE = B_LOADS / 4;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
    uint32_t a_voff[A_PER_WAVE];
#pragma unroll
    for (int q = 0; q < A_PER_WAVE; ++q) {
        const int c = w + 4 * q;
        const int iblk = c >> 1, h = c & 1;
        int row = iblk * 16 + li;
        if (GENERIC) row = (m0 + row < M) ? row : (M - 1 - m0);
        a_voff[q] = (uint32_t)(((int64_t)row * lda + E * (4 * h + lg)) * SZ);
    }
    const uint32_t b_voff = (uint32_t)((((int64_t)(l / LPR)) * ldb + E * (l % LPR)) * SZ);
    const char *const a_base = reinterpret_cast<const char *>(A + (int64_t)m0 * lda);
    const char *const b_base = reinterpret_cast<const char *>(B + n0);
    auto fetch_async_a = [&](int kt, int buf) {
        const uint32_t dst = lds_base + buf * STAGE + w * 1024;
        const char *src = a_base + (int64_t)kt * (BK * SZ);
#pragma unroll
        for (int q = 0; q < A_PER_WAVE; ++q) async_copy16(a_voff[q], src, dst + q * 4096);
    };
    auto fetch_async_b = [&](int kt, int buf) {
        // load r = w + 4q starts at row r * RPI = w * RPI + q * (4 * RPI); 4 * RPI is a multiple of E,
        // so q only moves the destination by whole groups
        const int64_t row_bytes = ldb * SZ;
        const uint32_t dst0 = lds_base + buf * STAGE + A_STAGE + ((w * RPI) / E) * B_GROUP + ((w * RPI) % E) * B_ROW;
        const char *src0 = b_base + (int64_t)(kt * BK + w * RPI) * row_bytes;
        constexpr int Q_GROUPS = (4 * RPI) / E;
        static_assert((4 * RPI) % E == 0, "loads of one wave are whole groups apart");
        if (!b_edge) {
#pragma unroll
            for (int q = 0; q < B_PER_WAVE; ++q)
                async_copy16(b_voff, src0 + (int64_t)(4 * RPI * q) * row_bytes, dst0 + q * Q_GROUPS * B_GROUP);
        } else {
            const int valid = N - n0;                      // 1 .. BN-1 columns of this tile exist
            const bool cell_ok = E * (l % LPR) + E <= valid;
            const int jt = (valid / E) * E;                // first column of a partly valid cell
            const int tail_dwords = (valid % E) * (SZ / 4);
#pragma unroll
            for (int q = 0; q < B_PER_WAVE; ++q) {
                const char *src = src0 + (int64_t)(4 * RPI * q) * row_bytes;
                const uint32_t dst = dst0 + q * Q_GROUPS * B_GROUP;
                if (cell_ok) async_copy16(b_voff, src, dst);
                if (l < tail_dwords) {
#pragma unroll
                    for (int rr = 0; rr < RPI; ++rr)
                        async_copy4(4 * l, src + rr * row_bytes + jt * SZ, dst + rr * B_ROW + jt * SZ);
                }
            }
        }
    };

    // ---- VGPR path (ragged K, unaligned operands): element-wise loads, zero outside the logical
    // matrices, written to LDS in the same layout.  Both operands are zeroed for k >= K, so padding
    // only ever forms 0 * 0.
    auto load_regs_a = [&](int kt, T (&ra)[E * NA]) {
        const int k0 = kt * BK;
#pragma unroll
        for (int q = 0; q < NA; ++q) {
            const int row = m0 + li + 16 * w + 64 * (q >> 1), k = k0 + E * (lg + 4 * (q & 1));
            const T *p = A + (int64_t)row * lda + k;
#pragma unroll
            for (int e = 0; e < E; ++e) ra[E * q + e] = (row < M && k + e < K) ? p[e] : T(0);
        }
    };
    auto store_regs_a = [&](int buf, const T (&ra)[E * NA]) {
        char *stage = lds + buf * STAGE;
#pragma unroll
        for (int q = 0; q < NA; ++q) {
            const int i = li + 16 * w + 64 * (q >> 1), kc = lg + 4 * (q & 1);
            cell_t v;
#pragma unroll
            for (int e = 0; e < E; ++e) v[e] = ra[E * q + e];
            *reinterpret_cast<cell_t *>(stage + (((i >> 4) << 1) | (kc >> 2)) * 1024 + (kc & 3) * 256 + (i & 15) * 16) = v;
        }
    };
    auto load_regs_b = [&](int kt, T (&rb)[E * NB]) {
        const int k0 = kt * BK;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int kk = k0 + l / CPR + (64 / CPR) * w + (kThreads / CPR) * q, col = n0 + E * (l % CPR);
            const T *p = B + (int64_t)kk * ldb + col;
#pragma unroll
            for (int e = 0; e < E; ++e) rb[E * q + e] = (kk < K && col + e < N) ? p[e] : T(0);
        }
    };
    auto store_regs_b = [&](int buf, const T (&rb)[E * NB]) {
        char *stage = lds + buf * STAGE;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int kk = l / CPR + (64 / CPR) * w + (kThreads / CPR) * q, jc = l % CPR;
            cell_t v;
#pragma unroll
            for (int e = 0; e < E; ++e) v[e] = rb[E * q + e];
            *reinterpret_cast<cell_t *>(stage + A_STAGE + (kk / E) * B_GROUP + (kk % E) * B_ROW + jc * 16) = v;
        }
    };
    auto fetch_sync = [&](int kt, int buf) {
        T ra[E * NA];
        load_regs_a(kt, ra);
        store_regs_a(buf, ra);
        T rb[E * NB];
        load_regs_b(kt, rb);
        store_regs_b(buf, rb);
    };
    // kStaged: the registers that carry a stage from its loads (after one barrier) to its LDS
    // writes (before the next)
    T sa[STAGED ? E * NA : 1], sb[STAGED ? E * NB : 1];
    (void)sa;
    (void)sb;
    // issue what can be fetched asynchronously for stage kt (as early as its buffer is free) ...
    auto fetch_early = [&](int kt, int buf) {
        if (kt < nk_async) {
            fetch_async_a(kt, buf);
            fetch_async_b(kt, buf);
        }
    };
    // ... and fetch the rest synchronously just before the barrier that publishes the stage
    auto fetch_late = [&](int kt, int buf) {
        if (GENERIC && kt >= nk_async) fetch_sync(kt, buf);
    };

    // ---- operand fragments: one half-stage (h) = E MFMA k-steps -------------------------------
    const int a_frag = ((wm * (TM / 16)) << 1) * 1024 + l * 16;              // + mi*2048 + h*1024
    const int b_frag = A_STAGE + lg * B_GROUP + (wn * TN + li) * SZ;         // + h*4*B_GROUP + ni*16*SZ + e*B_ROW
    auto read_frags = [&](int buf, int h, cell_t (&fa)[MI], cell_t (&fb)[NI]) {
        const char *stage = lds + buf * STAGE;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
            fa[mi] = *reinterpret_cast<const cell_t *>(stage + a_frag + mi * 2048 + h * 1024);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const char *p = stage + b_frag + h * 4 * B_GROUP + ni * 16 * SZ;
#pragma unroll
            for (int e = 0; e < E; ++e) fb[ni][e] = *reinterpret_cast<const T *>(p + e * B_ROW);
        }
    };

    acc_t acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = acc_t{T(0), T(0), T(0), T(0)};

    // MFMAs lo .. hi-1 of the E * MI * NI that consume one half-stage, in the order e, mi, ni
    constexpr int HALF = E * MI * NI;
    auto mfma_range = [&](const cell_t (&fa)[MI], const cell_t (&fb)[NI], int lo, int hi) {
#pragma unroll
        for (int idx = 0; idx < HALF; ++idx) {
            if (idx < lo || idx >= hi) continue;
            const int e = idx / (MI * NI), mi = (idx / NI) % MI, ni = idx % NI;
            acc[mi][ni] = EL::mfma(fa[mi][e], fb[ni][e], acc[mi][ni]);
        }
    };

    cell_t fa0[MI], fb0[NI], fa1[MI], fb1[NI];

    // prologue: stages 0 and 1
    for (int kt = 0; kt < 2 && kt < nk; ++kt) {
        if (STAGED) fetch_sync(kt, kt);
        else {
            fetch_early(kt, kt);
            fetch_late(kt, kt);
        }
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
                store_regs_a(cur ^ 1, reinterpret_cast<const T(&)[E * NA]>(sa));
                store_regs_b(cur ^ 1, reinterpret_cast<const T(&)[E * NB]>(sb));
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
                load_regs_a(s + 2, reinterpret_cast<T(&)[E * NA]>(sa));
                load_regs_b(s + 2, reinterpret_cast<T(&)[E * NB]>(sb));
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
    const int row_base = m0 + wm * TM;
    const int col_base = n0 + wn * TN + li;
    constexpr int MB = (MI >= 2) ? 2 : 1;
#pragma unroll
    for (int mb = 0; mb < MI; mb += MB) {
        T cin[MB][NI][4];
#pragma unroll
        for (int mi = mb; mi < mb + MB; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = row_base + mi * 16 + EL::d_row(r, lg), col = col_base + ni * 16;
                    if (!GENERIC || tile_full || (row < M && col < N)) cin[mi - mb][ni][r] = C[(int64_t)row * ldc + col];
                    else cin[mi - mb][ni][r] = T(0);
                }
#pragma unroll
        for (int mi = mb; mi < mb + MB; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = row_base + mi * 16 + EL::d_row(r, lg), col = col_base + ni * 16;
                    if (!GENERIC || tile_full || (row < M && col < N))
                        C[(int64_t)row * ldc + col] = cin[mi - mb][ni][r] + acc[mi][ni][r];
                }
    }
}

// Reference-shaped kernel without tiling or staging: one thread per element of C, k ascending.
// Kept as the bottom rung of the ladder (the paper's Section 2.3 starting point) and as an
// on-device cross-check that shares nothing with the MFMA kernel.
template <typename T>
__global__ void __launch_bounds__(256)
gemm_naive_kernel(int M, int N, int K, const T *__restrict__ A, int64_t lda, const T *__restrict__ B, int64_t ldb,
                  T *__restrict__ C, int64_t ldc)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)M * N) return;
    const int i = (int)(idx / N), j = (int)(idx % N);
    T c = C[(int64_t)i * ldc + j];
    const T *a = A + (int64_t)i * lda;
    for (int k = 0; k < K; ++k) c += a[k] * B[(int64_t)k * ldb + j];
    C[(int64_t)i * ldc + j] = c;
}

}  // namespace gemm_detail
