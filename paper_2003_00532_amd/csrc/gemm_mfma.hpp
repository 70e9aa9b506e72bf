// MFMA GEMM kernels for gfx950 (MI355X): C += A * B, and the full C <- alpha * op(A) * op(B) + beta * C,
// row-major, for double and float elements.
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
// v_mfma_f32_32x32x2_f32 takes A (i = l % 32, k = l / 32), B (k = l / 32, j = l % 32) and returns sixteen elements per
// lane, register r holding (i = 8 * (r / 4) + 4 * (l / 32) + r % 4, j = l % 32).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace gemm_detail {

typedef double v4d __attribute__((ext_vector_type(4)));
typedef double v2d __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kXcds = 8;    // workgroups are dealt round-robin to 8 XCDs, each with a private L2
constexpr int kGroupM = 8;  // tile rows per group of the grouped tile order
constexpr int kThreads = 256;
constexpr int kLean = 0, kGeneric = 1, kStaged = 2, kSampled = 3;  // kernel modes, see gemm_mfma_kernel

// What depends on the element type and on the matrix instruction.  A 16-byte LDS cell holds E consecutive k (for A)
// of one row; one LDS stage is 8 cells deep, so BK = 8 * E (16 for double, 32 for float).  The instruction works on
// BLK x BLK blocks of C: lane l supplies one element of each operand, (x = l % BLK, k-lane kl = l / BLK), so one
// instruction consumes KL = 64 / BLK values of k, and returns ACC elements of the block per lane, register r holding
// row d_row(r, l), column l % BLK.  A half-stage is four cells deep; a lane reads cell KL * rr + kl of it for
// rr = 0 .. RPH-1 (RPH = 4 / KL reads per block and half-stage) and each read feeds E instructions.
//   double: v_mfma_f64_16x16x4_f64 (64 cycles), the only shape with full rate.
//   float:  v_mfma_f32_16x16x4_f32 (32 cycles); v_mfma_f32_32x32x2_f32 (64 cycles: the instruction count and issue
//           pattern per flop of the double kernel) is an option of the build that was measured and is not used, see
//           gemm_mfma_kernel.
template <typename T, int BLK> struct Elem;
template <> struct Elem<double, 16> {
    static constexpr int E = 2, BLK = 16, KL = 4, RPH = 1, ACC = 4;
    typedef v2d cell_t;
    typedef v4d acc_t;
    static __device__ __forceinline__ acc_t mfma(double a, double b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    static constexpr __device__ __forceinline__ int d_row(int r, int kl) { return 4 * r + kl; }
};
template <> struct Elem<float, 16> {
    static constexpr int E = 4, BLK = 16, KL = 4, RPH = 1, ACC = 4;
    typedef v4f cell_t;
    typedef v4f acc_t;
    static __device__ __forceinline__ acc_t mfma(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static constexpr __device__ __forceinline__ int d_row(int r, int kl) { return 4 * kl + r; }
};
template <> struct Elem<float, 32> {
    static constexpr int E = 4, BLK = 32, KL = 2, RPH = 2, ACC = 16;
    typedef v4f cell_t;
    typedef v16f acc_t;
    static __device__ __forceinline__ acc_t mfma(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    // four groups of four consecutive rows, 8 rows apart; the two k-lanes interleave them
    static constexpr __device__ __forceinline__ int d_row(int r, int kl) { return 8 * (r / 4) + 4 * kl + r % 4; }
};

// Split K: a launch of grid height S computes S consecutive slices of the k range, slice y into its own
// output slab, to be summed afterwards.  k_chunk is the slice length (a multiple of the stage depth, or K
// itself when nothing is split); the steps are what slice y adds, in elements, to the three base pointers.
struct SplitK {
    int k_chunk;
    int64_t step_a, step_b, step_c;
    int flags = 0;   // kFlag* bits
};
constexpr int kFlagAtomicC = 1;   // alpha = beta = 1: add the sums to C in memory instead of load, add, store

// Elements between neighbours along the contiguous index of op(A) and op(B) and along the rows of C; read by the
// kSampled mode only (1 everywhere else).
struct ElemStrides {
    int64_t a, b, c;
};

// Optional phase trace (diagnostic builds only, -DGEMM_PHASE_TRACE; driven by paper_2003_00532_amd/phase_trace.py):
// wave 0 of every workgroup stores the constant 100 MHz clock at a few points of its life (slots 0, 3, 4, 5: entry,
// after the first stage barrier, after the K loop, exit), the shader clock at entry and exit (slots 1, 2) and where
// it ran (slot 7), into 8 slots of a buffer the host has installed.
#ifdef GEMM_PHASE_TRACE
static __device__ unsigned long long *g_phase_trace;
#define GEMM_PHASE_MARK(i)                                                                                      \
    do {                                                                                                        \
        if (__builtin_amdgcn_readfirstlane(threadIdx.x >> 6) == 0 && g_phase_trace)                             \
            g_phase_trace[((size_t)blockIdx.x + (size_t)gridDim.x * blockIdx.y) * 8 + (i)] = __builtin_amdgcn_s_memrealtime(); \
    } while (0)
#define GEMM_PHASE_CLOCK(i)                                                                                     \
    do {                                                                                                        \
        if (__builtin_amdgcn_readfirstlane(threadIdx.x >> 6) == 0 && g_phase_trace)                             \
            g_phase_trace[((size_t)blockIdx.x + (size_t)gridDim.x * blockIdx.y) * 8 + (i)] = __builtin_amdgcn_s_memtime(); \
    } while (0)
#define GEMM_PHASE_WHERE()                                                                                      \
    do {                                                                                                        \
        if (__builtin_amdgcn_readfirstlane(threadIdx.x >> 6) == 0 && g_phase_trace)                             \
            g_phase_trace[((size_t)blockIdx.x + (size_t)gridDim.x * blockIdx.y) * 8 + 7] =                      \
                (unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 4) |                                 \
                ((unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 20) << 32);                         \
    } while (0)
#else
#define GEMM_PHASE_MARK(i) do { } while (0)
#define GEMM_PHASE_CLOCK(i) do { } while (0)
#define GEMM_PHASE_WHERE() do { } while (0)
#endif

// Division of a non-negative 32-bit number by a divisor fixed on the host, as a multiplication and a shift: the
// quotient is exact for every n < 2^31.  With L = ceil(log2 d) and m = floor(2^(31+L) / d) + 1 (which fits in 32 bits
// because d > 2^(L-1)), n * m / 2^(31+L) exceeds n / d by less than n / 2^(31+L) < 2^-L <= 1/d, so the floor is the
// same.  On the device every operand is wave-uniform and the whole computation stays on the scalar unit: a division
// by a run-time value would instead go through the vector unit's reciprocal, where, in a workgroup that starts while
// older ones are in their K loops, each instruction queues behind the matrix instructions of those waves.
struct FastDiv {
    uint32_t d, magic, shift;
};

inline FastDiv make_fast_div(uint32_t d)
{
    if (d <= 1) return FastDiv{1, 0, 0};
    uint32_t L = 0;
    while (((uint64_t)1 << L) < d) ++L;   // ceil(log2 d) >= 1
    return FastDiv{d, (uint32_t)((((uint64_t)1 << (31 + L)) / d) + 1), L - 1};
}

__host__ __device__ inline uint32_t fast_div(uint32_t n, const FastDiv &f)
{
#ifdef __HIP_DEVICE_COMPILE__
    const uint32_t hi = __umulhi(n, f.magic);
#else
    const uint32_t hi = (uint32_t)(((uint64_t)n * f.magic) >> 32);
#endif
    return f.d == 1 ? n : (hi >> f.shift);
}

// Workgroup id -> tile coordinates.  Block b runs on XCD b % kXcds.  Each XCD receives a
// contiguous run of the "grouped" tile order (kGroupM tile rows at a time, column by column
// inside a group), so the workgroups resident on one XCD at any moment form a compact patch of C
// and re-use each other's A and B panels in that XCD's L2.
// All quantities fit in 32 bits: the host refuses problems with more than 2^31 - 1 blocks of 256 outputs.
// The host prepares what does not depend on the block (TileMap); the two divisions by run-time values (by the
// tiles of a group, and by the height of the last, shorter group) are FastDiv multiplications.
struct TileMap {
    uint32_t tiles_m, tiles_n;
    uint32_t per, rem;     // tiles per XCD and how many XCDs get one more
    FastDiv width;         // tiles in a full group of kGroupM tile rows
    FastDiv last;          // height of the last group (tiles_m % kGroupM, or kGroupM)
};

// `blocks` is the number of leading positions of the order that are dealt to the XCDs this way (all of them, unless
// the last ones are computed in slices, see TailSplit).
inline TileMap make_tile_map(uint32_t tiles_m, uint32_t tiles_n, uint32_t blocks = 0)
{
    const uint32_t total = blocks ? blocks : tiles_m * tiles_n;
    const uint32_t last = tiles_m % kGroupM ? tiles_m % kGroupM : kGroupM;
    return TileMap{tiles_m, tiles_n, total / kXcds, total % kXcds, make_fast_div(kGroupM * tiles_n), make_fast_div(last)};
}

// Position, in the grouped order, of the tile of workgroup b.
__host__ __device__ inline uint32_t position_of_block(uint32_t b, const TileMap &map)
{
    static_assert(kXcds == 8 && kGroupM == 8, "the shifts below");
    const uint32_t x = b & 7, s = b >> 3;
    const uint32_t start = x * map.per + (x < map.rem ? x : map.rem);
    return start + s;
}

// Tile coordinates of position `logical` of the grouped order.
__host__ __device__ inline void tile_at(uint32_t logical, const TileMap &map, uint32_t &tm, uint32_t &tn)
{
    const uint32_t g = fast_div(logical, map.width);
    const uint32_t first_m = g * kGroupM;
    const bool full = map.tiles_m - first_m >= (uint32_t)kGroupM;
    const uint32_t gsz = full ? (uint32_t)kGroupM : map.tiles_m - first_m;
    const uint32_t in_g = logical - g * map.width.d;
    tn = full ? (in_g >> 3) : fast_div(in_g, map.last);
    tm = first_m + (in_g - tn * gsz);
}

__host__ __device__ inline void tile_of_block(uint32_t b, const TileMap &map, uint32_t &tm, uint32_t &tn)
{
    tile_at(position_of_block(b, map), map, tm, tn);
}

// Tail split.  A launch whose tiles do not fill the chip's workgroup slots in whole rounds leaves the last, partial
// round to a few compute units.  With a workspace the host can cut the k range of just those last tiles: blocks
// 0 .. begin-1 compute whole tiles as usual (positions 0 .. begin-1 of the grouped order), and every later block is
// one slice of one of the remaining tiles: unit u = block - begin computes slice u % S of the tile at position
// begin + u / S into its own dense BM x BN slab, slab u of `slabs`; a second launch adds the slabs of each tile in
// ascending order and applies alpha, beta (tail_reduce_kernel).  begin == UINT32_MAX: no tail.
struct TailSplit {
    uint32_t begin;
    FastDiv splits;            // S
    int k_chunk;               // slice length, a multiple of the stage depth
    int64_t step_a, step_b;    // what one slice adds, in elements, to the pointers of A and B
    void *slabs;
};
inline TailSplit no_tail() { return TailSplit{UINT32_MAX, FastDiv{1, 0, 0}, 0, 0, 0, nullptr}; }

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
// Completion is awaited by the s_waitcnt vmcnt(0) inside stage_barrier().  The statement writes M0 (the
// LDS destination of the copy) and says so in its clobber list.
__device__ __forceinline__ void async_copy16(uint32_t voff, const void *sbase, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(voff), "s"(sbase), "s"(lds_addr)
                 : "memory", "m0");
}

// The 4-byte form: lane l copies the 4 bytes at sbase + voff(l) to LDS address lds_addr + 4 * l.
__device__ __forceinline__ void async_copy4(uint32_t voff, const void *sbase, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :
                 : "v"(voff), "s"(sbase), "s"(lds_addr)
                 : "memory", "m0");
}

// The scalar tail of C <- alpha * s + beta * c: t = alpha * s, then t itself when beta is zero (c is
// not used), else t + beta * c, every operation rounded on its own (no fused multiply-add), so that
// the tail is the same sequence of roundings as a term-by-term evaluation; with alpha = beta = 1 both
// products are exact and what is left is the single rounding of s + c.
template <typename T>
__device__ __forceinline__ T scaled_update(T alpha, T s, T beta, T c, bool read_c)
{
#pragma clang fp contract(off)
    const T t = alpha * s;
    if (!read_c) return t;
    const T u = beta * c;
    return t + u;
}

// One operand panel of the macro-tile: how a BX x BK slice (BX = BM rows of op(A), or BN columns of
// op(B)) is fetched from memory, laid out in LDS and read back as MFMA operand fragments.  The two MFMA
// operands are symmetric (lane l supplies element (x = l % 16, k = l / 16) of either), so what matters is
// only which index is contiguous in memory:
//
//   KMAJOR (k contiguous: A as given, or a transposed B stored N x K): element (x, k) at P[x * ld + k].
//      LDS: 1 KiB chunks indexed [x / 16][h], h = kc / 4 with kc = k / E the cell index along k; inside a
//      chunk the 16-byte cell of lane-slot (kq, xx), kq = kc % 4, xx = x % 16, sits at (kq * 16 + xx) * 16
//      and holds E consecutive k.  A wave's operand fetch for one 16-wide block and one h is a single
//      1 KiB lane-linear ds_read_b128, and its E elements feed E MFMA k-steps: step e uses
//      k = E * (4h + l/16) + e in lane group l/16.
//   not KMAJOR (x contiguous: B as given, or a transposed A stored K x M): element (x, k) at P[k * ld + x].
//      LDS: groups of E rows [k / E] at a stride of E*BX*sizeof(T) + 16*sizeof(T) bytes, the rows of a
//      group BX*sizeof(T) apart; a lane reads rows E*(4h + l/16) + e, e = 0..E-1, at its own x: the same
//      k per step as above.  The group stride is 16*sizeof(T) modulo 256 bytes, so the 16-lane groups
//      that are served together fall into different banks.
//
// Both layouts are exactly what a 16-byte-per-lane global->LDS load writes (lane-linear 1 KiB), so
// full panels are staged with global_load_lds_dwordx4 and never pass through VGPRs.  Every address of
// that path is a wave-uniform 64-bit base, advanced with scalar arithmetic, plus a 32-bit per-lane
// byte offset computed once: MFMAs and ordinary vector ALU instructions compete for the same issue
// cycles on this chip, so the K loop should contain none of the latter.  (The host only selects the
// path when 128 * ld, in bytes, fits in 32 bits.)  The copies need the global address aligned to the
// element only, not to their own 16 bytes.
//
// Edges along x (GENERIC only).  KMAJOR: rows at or beyond the extent X are redirected to row X - 1;
// they only feed outputs that are never stored, so no zero fill is needed and such tiles stay on the
// asynchronous path.  Not KMAJOR: lanes whose cell of E columns lies outside are switched off (their
// LDS cells keep stale bits, which again only feed outputs never stored) and a partly valid last cell
// is fetched on its own, four bytes per lane.
//
// The VGPR path (load_regs / store_regs: ragged last K stage, very large leading dimensions, operands sampled
// with a stride in both directions) loads element-wise, with zeros outside the logical matrix, and writes the
// same LDS layout.  Both operands are zeroed for k >= K, so padding only ever forms 0 * 0.  Only this path
// knows an element stride `es` along the contiguous index: element (x, k) sits at P[x * ld + k * es]
// (KMAJOR) or P[k * ld + x * es]; the asynchronous copies need es == 1, and every mode but kSampled passes
// the literal 1.
template <typename T, bool KMAJOR, int BX, bool GENERIC>
struct Panel {
    typedef Elem<T, 16> EL;   // the cell is the same for every instruction shape
    typedef typename EL::cell_t cell_t;
    static constexpr int E = EL::E;
    static constexpr int SZ = (int)sizeof(T);
    static constexpr int BK = 8 * E;
    // 32-wide panels exist for the k-contiguous kind only (a 1 KiB load of the other kind would span two
    // groups of rows)
    static_assert(BX == 64 || BX == 128 || (BX == 32 && KMAJOR), "supported panel widths");
    // KMAJOR
    static constexpr int CHUNKS = (BX / 16) * 2;
    static constexpr int CHUNKS_PER_WAVE = CHUNKS / 4;
    // not KMAJOR
    static constexpr int ROW = BX * SZ;                // bytes between consecutive k rows of a group
    static constexpr int GROUP = E * ROW + 16 * SZ;    // bytes between groups of E rows
    static_assert(GROUP % 256 == 16 * SZ, "group stride must be 16 elements modulo 256 bytes");
    static constexpr int LOADS = (BK * BX * SZ) / 1024;  // 1 KiB global->LDS loads per stage
    static constexpr int LOADS_PER_WAVE = LOADS / 4;
    static constexpr int RPI = 1024 / ROW;             // k rows covered by one such load
    static constexpr int LPR = 64 / RPI;               // lanes per row in it
    static_assert(KMAJOR || (RPI >= 1 && RPI <= E && E % RPI == 0), "a load stays inside one group of rows");
    static constexpr int Q_GROUPS = (4 * RPI) / E;
    static_assert(KMAJOR || (4 * RPI) % E == 0, "loads of one wave are whole groups apart");
    static constexpr int CPR = BX / E;                 // cells per k row
    static_assert(64 % CPR == 0, "a wave covers whole rows of cells");

    static constexpr int STAGE_BYTES = KMAJOR ? CHUNKS * 1024 : 8 * GROUP;
    static constexpr int NR = BX / 32;                 // 16-byte cells per thread per stage on the VGPR path
    // VGPR path, k-contiguous kind: which cell (row in the panel, cell index along k) thread (w, lg, li)
    // handles as its q-th; 256 threads cover 32 rows x 8 cells at a time
    __device__ __forceinline__ int vg_row(int q) const { return BX == 32 ? li + 16 * (w & 1) : li + 16 * w + 64 * (q >> 1); }
    __device__ __forceinline__ int vg_cell(int q) const { return BX == 32 ? lg + 4 * (w >> 1) : lg + 4 * (q & 1); }

    const T *P;
    int64_t ld;
    int64_t es;   // elements between neighbours along the panel's contiguous index; other than 1 on the VGPR path only
    int x0, X, K;
    int w, l, lg, li;
    uint32_t voff[KMAJOR ? CHUNKS_PER_WAVE : 1];
    const char *base;
    bool edge;

    __device__ __forceinline__ void init(const T *P_, int64_t ld_, int64_t es_, int x0_, int X_, int K_, int w_, int l_)
    {
        P = P_; ld = ld_; es = es_; x0 = x0_; X = X_; K = K_; w = w_; l = l_;
        lg = l >> 4; li = l & 15;
        edge = GENERIC && (x0 + BX > X);
        if constexpr (KMAJOR) {
            // chunk c = (blk, h): lane l fetches the cell (row blk*16 + l%16, cell 4h + l/16 along k)
#pragma unroll
            for (int q = 0; q < CHUNKS_PER_WAVE; ++q) {
                const int c = w + 4 * q;
                const int blk = c >> 1, h = c & 1;
                int row = blk * 16 + li;
                if (GENERIC) row = (x0 + row < X) ? row : (X - 1 - x0);
                voff[q] = (uint32_t)(((int64_t)row * ld + E * (4 * h + lg)) * SZ);
            }
            base = reinterpret_cast<const char *>(P + (int64_t)x0 * ld);
        } else {
            // load r covers k rows r*RPI .. r*RPI + RPI-1: lane l fetches row r*RPI + l/LPR, cell l%LPR
            voff[0] = (uint32_t)((((int64_t)(l / LPR)) * ld + E * (l % LPR)) * SZ);
            base = reinterpret_cast<const char *>(P + x0);
        }
    }

    // each wave issues its share of the 1 KiB global->LDS loads of stage kt; `dst` is the LDS byte
    // address of this panel in the destination stage buffer
    __device__ __forceinline__ void fetch_async(int kt, uint32_t dst) const
    {
        if constexpr (KMAJOR) {
            const char *src = base + (int64_t)kt * (BK * SZ);
#pragma unroll
            for (int q = 0; q < CHUNKS_PER_WAVE; ++q) async_copy16(voff[q], src, dst + w * 1024 + q * 4096);
        } else {
            // load r = w + 4q starts at k row r * RPI = w * RPI + q * (4 * RPI); 4 * RPI is a multiple
            // of E, so q only moves the destination by whole groups
            const int64_t row_bytes = ld * SZ;
            const uint32_t dst0 = dst + ((w * RPI) / E) * GROUP + ((w * RPI) % E) * ROW;
            const char *src0 = base + (int64_t)(kt * BK + w * RPI) * row_bytes;
            if (!edge) {
#pragma unroll
                for (int q = 0; q < LOADS_PER_WAVE; ++q)
                    async_copy16(voff[0], src0 + (int64_t)(4 * RPI * q) * row_bytes, dst0 + q * Q_GROUPS * GROUP);
            } else {
                const int valid = X - x0;                      // 1 .. BX-1 columns of this panel exist
                const bool cell_ok = E * (l % LPR) + E <= valid;
                const int xt = (valid / E) * E;                // first column of a partly valid cell
                const int tail_dwords = (valid % E) * (SZ / 4);
#pragma unroll
                for (int q = 0; q < LOADS_PER_WAVE; ++q) {
                    const char *src = src0 + (int64_t)(4 * RPI * q) * row_bytes;
                    const uint32_t d = dst0 + q * Q_GROUPS * GROUP;
                    if (cell_ok) async_copy16(voff[0], src, d);
                    if (l < tail_dwords) {
#pragma unroll
                        for (int rr = 0; rr < RPI; ++rr)
                            async_copy4(4 * l, src + rr * row_bytes + xt * SZ, d + rr * ROW + xt * SZ);
                    }
                }
            }
        }
    }

    __device__ __forceinline__ void load_regs(int kt, T (&r)[E * NR]) const
    {
        const int k0 = kt * BK;
#pragma unroll
        for (int q = 0; q < NR; ++q) {
            if constexpr (KMAJOR) {
                const int row = x0 + vg_row(q), k = k0 + E * vg_cell(q);
                const T *p = P + (int64_t)row * ld + k * es;
#pragma unroll
                for (int e = 0; e < E; ++e) r[E * q + e] = (row < X && k + e < K) ? p[e * es] : T(0);
            } else {
                const int kk = k0 + l / CPR + (64 / CPR) * w + (kThreads / CPR) * q, col = x0 + E * (l % CPR);
                const T *p = P + (int64_t)kk * ld + col * es;
#pragma unroll
                for (int e = 0; e < E; ++e) r[E * q + e] = (kk < K && col + e < X) ? p[e * es] : T(0);
            }
        }
    }

    __device__ __forceinline__ void store_regs(char *stage, const T (&r)[E * NR]) const
    {
#pragma unroll
        for (int q = 0; q < NR; ++q) {
            cell_t v;
#pragma unroll
            for (int e = 0; e < E; ++e) v[e] = r[E * q + e];
            if constexpr (KMAJOR) {
                const int i = vg_row(q), kc = vg_cell(q);
                *reinterpret_cast<cell_t *>(stage + (((i >> 4) << 1) | (kc >> 2)) * 1024 + (kc & 3) * 256 + (i & 15) * 16) = v;
            } else {
                const int kk = l / CPR + (64 / CPR) * w + (kThreads / CPR) * q, xc = l % CPR;
                *reinterpret_cast<cell_t *>(stage + (kk / E) * GROUP + (kk % E) * ROW + xc * 16) = v;
            }
        }
    }

    // Byte offset, inside this panel's part of a stage, of the first fragment of the wave whose patch starts at
    // element wx_off of the panel, for an instruction on BLK-wide blocks: lane l supplies x = l % BLK at k-lane
    // kl = l / BLK (with BLK = 32 the two 16-row chunks of a block are addressed by bit 4 of the lane number).
    template <int BLK>
    __device__ __forceinline__ int frag_base(int wx_off) const
    {
        const int xr = l % BLK, kl = l / BLK;
        if constexpr (KMAJOR) return (((wx_off / 16) + (xr >> 4)) << 1) * 1024 + (kl * 16 + (xr & 15)) * 16;
        else return kl * GROUP + (wx_off + xr) * SZ;
    }

    // Fragments of one half-stage (h): for XI consecutive BLK-wide blocks, RPH reads each; read rr of a lane is cell
    // KL * rr + kl of the half-stage, whose E elements feed E MFMA k-steps.
    template <int XI, int BLK>
    static __device__ __forceinline__ void read_frags(const char *panel, int fbase, int h, cell_t (&f)[XI * (BLK / 16)])
    {
        constexpr int KL = 64 / BLK, RPH = 4 / KL;
        static_assert(RPH == BLK / 16, "reads per block");
#pragma unroll
        for (int xi = 0; xi < XI; ++xi) {
#pragma unroll
            for (int rr = 0; rr < RPH; ++rr) {
                if constexpr (KMAJOR) {
                    f[xi * RPH + rr] = *reinterpret_cast<const cell_t *>(panel + fbase + xi * (BLK / 16) * 2048 + h * 1024 + rr * KL * 256);
                } else {
                    const char *p = panel + fbase + h * 4 * GROUP + rr * KL * GROUP + xi * BLK * SZ;
#pragma unroll
                    for (int e = 0; e < E; ++e) f[xi * RPH + rr][e] = *reinterpret_cast<const T *>(p + e * ROW);
                }
            }
        }
    }
};

// One workgroup = 256 threads = 4 waves arranged WM x WN; each wave owns a (BM/WM) x (BN/WN)
// patch of the macro-tile as MI x NI accumulator tiles of 16 x 16.  One LDS stage holds BK = 8 * E
// values of k (16 for double, 32 for float) of the op(A) panel followed by the op(B) panel; see Panel
// for the layouts.  TA / TB say that A / B is stored transposed (K x M / N x K).
//
// MODE = kLean: every tile is full and K is a multiple of BK (checked on the host); only the
// asynchronous path is compiled in.
// MODE = kGeneric adds the element-wise, zero-filled path through VGPRs for the ragged last K stage
// (synchronous: once per tile; zeros are required there because k >= K contributes to every output)
// and handles edge tiles.
// MODE = kStaged sends every stage through VGPRs, loaded two stages ahead and written to LDS one stage
// ahead, at the price of 16 to 32 more live registers and of vector-ALU work in the K loop.  It
// addresses memory with 64-bit pointers and is what remains for leading dimensions too large for the
// 32-bit lane offsets of the asynchronous copies.
// MODE = kSampled is kStaged for operands whose elements are `es` apart along their contiguous index (a matrix
// sampled with a stride in both directions), C included; it is the only mode that reads `es`, and costs a
// few more registers, so it is built for the 64 x 64 tile only.
// (Asking the compiler for more than two waves per SIMD was measured to cost 3 to 25 % on the larger
// tiles: it then schedules the K loop differently; the smaller tiles fit more waves anyway.)
template <typename T, int BM, int BN, int WM, int WN, int MODE, bool TA, bool TB>
__global__ void __launch_bounds__(kThreads, 2)
gemm_mfma_kernel(int M, int N, int K_total, T alpha_, const T *__restrict__ A_, int64_t lda, const T *__restrict__ B_,
                 int64_t ldb, T beta_, T *__restrict__ C_, int64_t ldc_, TileMap map, SplitK split, ElemStrides es, TailSplit tail)
{
    GEMM_PHASE_MARK(0);
    GEMM_PHASE_CLOCK(1);
    GEMM_PHASE_WHERE();
    // What this workgroup computes: a whole tile (of slice blockIdx.y of k when the grid has a height), or, past
    // tail.begin, one k slice of one of the last tiles into its own slab (see TailSplit).  Everything here is
    // wave-uniform and stays on the scalar unit.
    // Every kernel argument the prologue needs is requested here, in one batch of scalar loads with one wait; left to
    // itself the compiler fetches them one dependent group after the other along the branches below.
    asm volatile("" ::"s"(A_), "s"(B_), "s"(C_), "s"(lda), "s"(ldb), "s"(ldc_), "s"(map.per), "s"(map.rem), "s"(map.width.magic),
                 "s"(map.width.shift), "s"(map.width.d), "s"(map.tiles_m), "s"(map.last.magic), "s"(map.last.shift), "s"(map.last.d),
                 "s"(split.k_chunk), "s"(tail.begin), "s"(K_total), "s"(M), "s"(N));
    const bool tail_unit = blockIdx.x >= tail.begin;
    uint32_t position;          // of the tile in the grouped order
    int slice, k_chunk;
    int64_t step_a, step_b;
    uint32_t unit = 0;
    T alpha = alpha_, beta = beta_;
    if (!tail_unit) {
        position = position_of_block(blockIdx.x, map);
        slice = (int)blockIdx.y;
        k_chunk = split.k_chunk;
        step_a = split.step_a;
        step_b = split.step_b;
    } else {
        unit = blockIdx.x - tail.begin;
        const uint32_t unit_tile = fast_div(unit, tail.splits);
        position = tail.begin + unit_tile;
        slice = (int)(unit - unit_tile * tail.splits.d);
        k_chunk = tail.k_chunk;
        step_a = tail.step_a;
        step_b = tail.step_b;
        alpha = T(1);
        beta = T(0);
    }
    const int K = min(k_chunk, K_total - slice * k_chunk);
    const T *__restrict__ A = A_ + slice * step_a;
    const T *__restrict__ B = B_ + slice * step_b;
    constexpr int TM = BM / WM, TN = BN / WN;
    // Single precision can also run on 32 x 32 blocks (-DGEMM_F32_WIDE_BLOCKS).  Measured on MI355X it is correct (the
    // whole float test-suite passes) and never faster: 8192^3 93.6 against 95.5 % of peak with the 128 x 128 tile, 93.0
    // against 96.2 % with 64 x 128, the same at 2048^3, with the same LDS instruction count, no bank conflicts and the
    // same matrix-pipe cycles in the counters; so the 16 x 16 instruction is what the library builds.
#ifdef GEMM_F32_WIDE_BLOCKS
    constexpr int BLK = (std::is_same<T, float>::value && TM % 32 == 0 && TN % 32 == 0) ? 32 : 16;
#else
    constexpr int BLK = 16;
#endif
    typedef Elem<T, BLK> EL;
    typedef typename EL::cell_t cell_t;
    typedef typename EL::acc_t acc_t;
    constexpr int E = EL::E, RPH = EL::RPH;
    constexpr int SZ = (int)sizeof(T);
    static_assert(E * SZ == 16, "a cell is 16 bytes");
    constexpr int BK = 8 * E;
    constexpr bool GENERIC = MODE != kLean;
    constexpr bool STAGED = MODE == kStaged || MODE == kSampled;
    constexpr bool SAMPLED = MODE == kSampled;
    static_assert(MODE == kLean || MODE == kGeneric || MODE == kStaged || MODE == kSampled, "kernel mode");
    static_assert(WM * WN == 4, "four waves per workgroup");
    constexpr int MI = TM / BLK, NI = TN / BLK;
    static_assert(MI >= 1 && NI >= 1 && TM % BLK == 0 && TN % BLK == 0, "wave tile is a grid of BLK x BLK blocks");
    typedef Panel<T, !TA, BM, GENERIC> PA;
    typedef Panel<T, TB, BN, GENERIC> PB;
    constexpr int A_STAGE = PA::STAGE_BYTES;
    constexpr int STAGE = A_STAGE + PB::STAGE_BYTES;
    constexpr int NA = PA::NR, NB = PB::NR;

    __shared__ __attribute__((aligned(1024))) char lds[2 * STAGE];

    const int t = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int l = t & 63;
    const int wm = w / WN, wn = w % WN;
    const int kl = l / BLK, lx = l % BLK;   // this lane's k-lane and its column inside a block of C

    uint32_t tm_u, tn_u;
    tile_at(position, map, tm_u, tn_u);
    const int m0 = (int)tm_u * BM, n0 = (int)tn_u * BN;
    // the output: C itself, or the slab of this unit addressed as if it were the tile's place in a matrix of BN columns
    const int64_t ldc = tail_unit ? (int64_t)BN : ldc_;
    T *__restrict__ C = tail_unit ? static_cast<T *>(tail.slabs) + (int64_t)unit * (BM * BN) - ((int64_t)m0 * BN + n0)
                                  : C_ + slice * split.step_c;

    const bool tile_full = (m0 + BM <= M) && (n0 + BN <= N);
    const int nk = (K + BK - 1) / BK;
    // number of leading stages fetched by the asynchronous global->LDS path; only the ragged last K
    // stage goes through VGPRs, for both operands
    const int nk_async = STAGED ? 0 : GENERIC ? K / BK : nk;

    PA pa;
    PB pb;
    pa.init(A, lda, SAMPLED ? es.a : 1, m0, M, K, w, l);
    pb.init(B, ldb, SAMPLED ? es.b : 1, n0, N, K, w, l);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;

    auto fetch_sync = [&](int kt, int buf) {
        T ra[E * NA];
        pa.load_regs(kt, ra);
        pa.store_regs(lds + buf * STAGE, ra);
        T rb[E * NB];
        pb.load_regs(kt, rb);
        pb.store_regs(lds + buf * STAGE + A_STAGE, rb);
    };
    // kStaged: the registers that carry a stage from its loads (after one barrier) to its LDS
    // writes (before the next)
    T sa[STAGED ? E * NA : 1], sb[STAGED ? E * NB : 1];
    (void)sa;
    (void)sb;
    // issue what can be fetched asynchronously for stage kt (as early as its buffer is free) ...
    auto fetch_early = [&](int kt, int buf) {
        if (kt < nk_async) {
            pa.fetch_async(kt, lds_base + buf * STAGE);
            pb.fetch_async(kt, lds_base + buf * STAGE + A_STAGE);
        }
    };
    // ... and fetch the rest synchronously just before the barrier that publishes the stage
    auto fetch_late = [&](int kt, int buf) {
        if (GENERIC && kt >= nk_async) fetch_sync(kt, buf);
    };

    // ---- operand fragments: one half-stage (h) = E MFMA k-steps -------------------------------
    const int a_frag = pa.template frag_base<BLK>(wm * TM);
    const int b_frag = A_STAGE + pb.template frag_base<BLK>(wn * TN);
    auto read_frags = [&](int buf, int h, cell_t (&fa)[MI * RPH], cell_t (&fb)[NI * RPH]) {
        const char *stage = lds + buf * STAGE;
        PA::template read_frags<MI, BLK>(stage, a_frag, h, fa);
        PB::template read_frags<NI, BLK>(stage, b_frag, h, fb);
    };

    // The accumulators are not cleared: the first MFMA into each of them (the first MI * NI of a tile's first
    // half-stage) takes a zero third operand instead, which the instruction accepts as a constant.  Clearing 64 to 128
    // registers per lane with moves costs a workgroup that starts under load one to three microseconds, because every
    // vector instruction of a young wave queues behind the matrix instructions of the older ones.
    acc_t acc[MI][NI];

    // MFMAs lo .. hi-1 of the RPH * E * MI * NI that consume one half-stage, in the order read, e, mi, ni (the
    // first ones only need the first read of every block)
    constexpr int HALF = RPH * E * MI * NI;
    auto mfma_range = [&](const cell_t (&fa)[MI * RPH], const cell_t (&fb)[NI * RPH], int lo, int hi, auto fresh_tag) {
        constexpr bool FRESH = decltype(fresh_tag)::value;   // the accumulators hold nothing yet
#pragma unroll
        for (int idx = 0; idx < HALF; ++idx) {
            if (idx < lo || idx >= hi) continue;
            const int rr = idx / (E * MI * NI), e = (idx / (MI * NI)) % E, mi = (idx / NI) % MI, ni = idx % NI;
            if (FRESH && idx < MI * NI) {
                acc_t zero;
#pragma unroll
                for (int r = 0; r < EL::ACC; ++r) zero[r] = T(0);
                acc[mi][ni] = EL::mfma(fa[mi * RPH + rr][e], fb[ni * RPH + rr][e], zero);
            } else {
                acc[mi][ni] = EL::mfma(fa[mi * RPH + rr][e], fb[ni * RPH + rr][e], acc[mi][ni]);
            }
        }
    };

    cell_t fa0[MI * RPH], fb0[NI * RPH], fa1[MI * RPH], fb1[NI * RPH];

    // prologue: stages 0 and 1
    for (int kt = 0; kt < 2 && kt < nk; ++kt) {
        if (STAGED) fetch_sync(kt, kt);
        else {
            fetch_early(kt, kt);
            fetch_late(kt, kt);
        }
    }
    stage_barrier();
    GEMM_PHASE_MARK(3);
    read_frags(0, 0, fa0, fb0);

    // Stage s lives in buffer s % 2.  Per iteration: the second half's fragments are read while the
    // first half's MFMAs run; then one barrier, after which buffer s % 2 is free for stage s + 2 and
    // stage s + 1 (fetched one iteration ago) is complete, so its first fragments are read and the
    // next fetch is issued underneath the second half's MFMAs.  The loop is unrolled by two so that
    // the buffer index is a compile-time constant and every LDS address is base register + immediate.
    // With two waves per SIMD (the 128 x 128 tile) a wave runs the MFMAs that lead up to its barrier at raised
    // priority and the ones after it at normal priority, so that the four waves of a workgroup arrive at the
    // barrier together while the other workgroup fills the gaps: +0.5 % at 8192^3.  With three or four waves
    // per SIMD the same scheme costs 2 to 5 %, so the smaller tiles leave priorities alone.
    constexpr bool RUSH_TO_BARRIER = BM * BN >= 128 * 128;
    auto iteration = [&](int s, auto cur_tag, auto fresh_tag) {
        constexpr int cur = decltype(cur_tag)::value;
        // The first MFMAs wait for fragments that were requested long ago; only then are the next
        // reads queued, so that wait never covers a read that has just been issued.
        if constexpr (RUSH_TO_BARRIER) __builtin_amdgcn_s_setprio(1);
        mfma_range(fa0, fb0, 0, NI, fresh_tag);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(cur, 1, fa1, fb1);
        __builtin_amdgcn_sched_barrier(0);
        mfma_range(fa0, fb0, NI, HALF, fresh_tag);
        if constexpr (STAGED) {
            if (s >= 1 && s + 1 < nk) {  // stage s + 1 was loaded during the previous iteration
                pa.store_regs(lds + (cur ^ 1) * STAGE, reinterpret_cast<const T(&)[E * NA]>(sa));
                pb.store_regs(lds + (cur ^ 1) * STAGE + A_STAGE, reinterpret_cast<const T(&)[E * NB]>(sb));
            }
        } else if (GENERIC && s >= 1 && s + 1 < nk) {
            fetch_late(s + 1, cur ^ 1);
        }
        stage_barrier();
        if constexpr (RUSH_TO_BARRIER) __builtin_amdgcn_s_setprio(0);
        // unconditional (in the last iteration it re-reads a stale buffer and the values are never
        // used): the number of LDS reads in flight is then the same on every path, and the compiler
        // waits for exactly the older ones before the MFMAs below instead of draining the queue
        read_frags(cur ^ 1, 0, fa0, fb0);
        if constexpr (STAGED) {
            if (s + 2 < nk) {
                pa.load_regs(s + 2, reinterpret_cast<T(&)[E * NA]>(sa));
                pb.load_regs(s + 2, reinterpret_cast<T(&)[E * NB]>(sb));
            }
        } else if (s + 2 < nk) {
            fetch_early(s + 2, cur);
        }
        __builtin_amdgcn_sched_barrier(0);
        mfma_range(fa1, fb1, 0, HALF, std::false_type{});
    };
    // C <- alpha * (A B) + beta * C, C read (unless beta is zero: then it may hold anything, NaN
    // included) and written exactly once per element, after the K loop.  With alpha = beta = 1 the
    // update is the single rounding of acc + c (see scaled_update).  Loads are issued in batches
    // of two 16-row blocks (up to 32 per lane in flight) before the first is consumed: the epilogue
    // is latency-bound, so its duration is the number of batches times the memory latency.
    // Addressing: one pointer per lane to its first element, then row steps of ROW_STEP * ldc elements
    // between the four result registers of an accumulator tile and 16 * ldc between tile rows, added up
    // as the loops go (a 64-bit add per row instead of a multiply per element); columns of one row are
    // a compile-time offset apart.
    auto write_tile = [&]() {
        // Result register r = 4 g + q of a block holds row d_row(r, kl): groups g of four registers ROW_STEP rows
        // apart, the groups GROUP_STEP rows apart (one group for the 16 x 16 instructions, four for 32 x 32).
        constexpr int ACC = EL::ACC, GROUPS = ACC / 4;
        constexpr int ROW_STEP = EL::d_row(1, 0) - EL::d_row(0, 0);   // 4 for double, 1 for float
        constexpr int GROUP_STEP = GROUPS > 1 ? EL::d_row(4 % ACC, 0) - EL::d_row(0, 0) : 0;
        static_assert(EL::d_row(2, 0) - EL::d_row(1, 0) == ROW_STEP && EL::d_row(3, 0) - EL::d_row(2, 0) == ROW_STEP, "");
        static_assert(GROUPS == 1 || EL::d_row(ACC - 4, 0) - EL::d_row(0, 0) == (GROUPS - 1) * GROUP_STEP, "");
        const int row_base = m0 + wm * TM + EL::d_row(0, kl);
        const int col_base = n0 + wn * TN + lx;
        constexpr int MB = (ACC == 4 && MI >= 2) ? 2 : 1;   // blocks of rows whose loads are in flight together
        const int64_t cs_c = SAMPLED ? es.c : 1;   // elements between neighbouring columns of C
        T *const c_lane = C + (int64_t)row_base * ldc + col_base * cs_c;
        const int64_t r_step = (int64_t)ROW_STEP * ldc, g_step = (int64_t)GROUP_STEP * ldc, mi_step = (int64_t)BLK * ldc;
        // Four forms, chosen once per workgroup: alpha = beta = 1 (the paper's own operation: one addition
        // per element) with the addition done by the lane or, on request of the host, by the memory system
        // (no-return floating-point atomics: each element belongs to one lane, so it is the same single rounding);
        // beta = 0 (C is not read); and the general one.
        constexpr int kUnit = 0, kOverwrite = 1, kScaled = 2, kUnitAtomic = 3;
        // visits every element (mi, ni, r) of the blocks mb .. mb + MB - 1 with its address and whether it exists
        auto for_each = [&](int mb, T *c_mb, auto &&body) {
            T *c_mi = c_mb;
#pragma unroll
            for (int mi = mb; mi < mb + MB; ++mi) {
#pragma unroll
                for (int g = 0; g < GROUPS; ++g) {
                    T *c_r = c_mi + g * g_step;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int r = 4 * g + q;
                        const int row = row_base + mi * BLK + g * GROUP_STEP + q * ROW_STEP;
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) {
                            const int col = col_base + ni * BLK;
                            body(mi, ni, r, &c_r[ni * BLK * cs_c], !GENERIC || tile_full || (row < M && col < N));
                        }
                        c_r += r_step;
                    }
                }
                c_mi += mi_step;
            }
        };
        auto epilogue = [&](auto kind_tag) {
            constexpr int KIND = decltype(kind_tag)::value;
            constexpr bool UNIT = KIND == kUnit;
            constexpr bool read_c = KIND != kOverwrite;
            T *c_mb = c_lane;
#pragma unroll
            for (int mb = 0; mb < MI; mb += MB) {
                if constexpr (KIND == kUnitAtomic) {
                    for_each(mb, c_mb, [&](int mi, int ni, int r, T *c, bool live) {
                        if (live) unsafeAtomicAdd(c, acc[mi][ni][r]);
                    });
                } else {
                    T cin[MB][NI][ACC];
                    for_each(mb, c_mb, [&](int mi, int ni, int r, T *c, bool live) {
                        cin[mi - mb][ni][r] = (read_c && live) ? *c : T(0);
                    });
                    for_each(mb, c_mb, [&](int mi, int ni, int r, T *c, bool live) {
                        if (live)
                            *c = UNIT ? cin[mi - mb][ni][r] + acc[mi][ni][r]
                                      : scaled_update(alpha, acc[mi][ni][r], beta, cin[mi - mb][ni][r], read_c);
                    });
                }
                c_mb += MB * mi_step;
            }
        };
        if (alpha == T(1) && beta == T(1) && (split.flags & kFlagAtomicC)) epilogue(std::integral_constant<int, kUnitAtomic>{});
        else if (alpha == T(1) && beta == T(1)) epilogue(std::integral_constant<int, kUnit>{});
        else if (beta == T(0)) epilogue(std::integral_constant<int, kOverwrite>{});
        else epilogue(std::integral_constant<int, kScaled>{});
    };

    // the first iteration is the one that meets fresh accumulators (nk >= 1: the host launches nothing for K == 0)
    iteration(0, std::integral_constant<int, 0>{}, std::true_type{});
    if (nk > 1) iteration(1, std::integral_constant<int, 1>{}, std::false_type{});
    int s = 2;
    for (; s + 1 < nk; s += 2) {
        iteration(s, std::integral_constant<int, 0>{}, std::false_type{});
        iteration(s + 1, std::integral_constant<int, 1>{}, std::false_type{});
    }
    if (s < nk) iteration(s, std::integral_constant<int, 0>{}, std::false_type{});
    GEMM_PHASE_MARK(4);
    write_tile();
    GEMM_PHASE_MARK(5);
    GEMM_PHASE_CLOCK(2);
}

// Reference-shaped kernel without tiling or staging: one thread per element of C, k ascending.
// Kept as the bottom rung of the ladder (the paper's Section 2.3 starting point), as an
// on-device cross-check that shares nothing with the MFMA kernel, and, since every operand is
// addressed through a row stride and a column stride (X(r, c) = X[r * rs + c * cs], the affine layout
// maps of Section 2.9), for any layout.
template <typename T>
__global__ void __launch_bounds__(256)
gemm_naive_kernel(int M, int N, int K, T alpha, const T *__restrict__ A, int64_t rsa, int64_t csa, const T *__restrict__ B,
                  int64_t rsb, int64_t csb, T beta, T *__restrict__ C, int64_t rsc, int64_t csc)
{
    // the grid may be smaller than the matrix (the runtime limits a launch to 2^32 threads): each thread strides on
    const int64_t total = (int64_t)M * N, step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += step) {
        const int i = (int)(idx / N), j = (int)(idx % N);
        const T *a = A + (int64_t)i * rsa, *b = B + (int64_t)j * csb;
        T acc = T(0);
        for (int k = 0; k < K; ++k) acc += a[k * csa] * b[k * rsb];
        const bool read_c = beta != T(0);
        T *c = C + (int64_t)i * rsc + (int64_t)j * csc;
        *c = scaled_update(alpha, acc, beta, read_c ? *c : T(0), read_c);
    }
}

// C <- beta * C (all zeros when beta is zero, whatever C held): what is left of the operation when
// alpha is zero or K is zero.
template <typename T>
__global__ void __launch_bounds__(256) scale_c_kernel(int M, int N, T beta, T *__restrict__ C, int64_t rsc, int64_t csc)
{
    const int64_t total = (int64_t)M * N, step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += step) {
        const int i = (int)(idx / N), j = (int)(idx % N);
        T *p = C + (int64_t)i * rsc + (int64_t)j * csc;
        *p = (beta != T(0)) ? beta * *p : T(0);
    }
}

// The second step of a split K: C <- alpha * (W_0 + W_1 + ... + W_{S-1}) + beta * C, the slabs W_p (M x N, dense)
// added in ascending p, so that the result does not depend on how the first step was scheduled.
template <typename T>
__global__ void __launch_bounds__(256)
split_k_reduce_kernel(int M, int N, int splits, T alpha, const T *__restrict__ W, T beta, T *__restrict__ C, int64_t ldc)
{
    const int64_t total = (int64_t)M * N, step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += step) {
        T s = W[idx];
        for (int p = 1; p < splits; ++p) s += W[p * total + idx];
        const int i = (int)(idx / N), j = (int)(idx % N);
        const bool read_c = beta != T(0);
        const T c = read_c ? C[(int64_t)i * ldc + j] : T(0);
        C[(int64_t)i * ldc + j] = scaled_update(alpha, s, beta, c, read_c);
    }
}

// The second step of a tail split (see TailSplit): for each of the last `tiles` tiles of the grouped order,
// C_tile <- alpha * (W_0 + ... + W_{S-1}) + beta * C_tile with the S slabs of the tile added in ascending order.
// One workgroup per 256 consecutive elements of a tile.
template <typename T>
__global__ void __launch_bounds__(256)
tail_reduce_kernel(int M, int N, int bm, int bn, TileMap map, uint32_t begin, int splits, T alpha, const T *__restrict__ W, T beta,
                   T *__restrict__ C, int64_t ldc)
{
    const int per_tile = bm * bn / 256;
    const uint32_t t = blockIdx.x / per_tile;
    const int e = (int)(blockIdx.x % per_tile) * 256 + (int)threadIdx.x;
    uint32_t tm, tn;
    tile_at(begin + t, map, tm, tn);
    const int i = (int)tm * bm + e / bn, j = (int)tn * bn + e % bn;
    if (i >= M || j >= N) return;
    const T *w = W + (int64_t)t * splits * (bm * bn) + e;
    T s = w[0];
    for (int p = 1; p < splits; ++p) s += w[(int64_t)p * (bm * bn)];
    const bool read_c = beta != T(0);
    T *c = C + (int64_t)i * ldc + j;
    *c = scaled_update(alpha, s, beta, read_c ? *c : T(0), read_c);
}

}  // namespace gemm_detail
