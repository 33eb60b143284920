// fp32 matrix-product kernels for gfx950 (CDNA4): 64-wide wavefronts, fp32 MFMA,
// operands staged through LDS.
//
// What is computed: C[i][j] = sum_k A[i][k] * opB[k][j] (Section 6.1 / 6.3 of the paper),
// fp32 in, fp32 accumulate on the matrix pipe, fp32 out.
//
// How the work is laid out (design for this chip, not the paper's CPU schedule):
//   * a workgroup owns a BM x BN tile of C and walks K in slabs of BK;
//   * each wave owns a (32*MB) x (32*NB) sub-tile held in MB*NB accumulators of the
//     32x32x2 fp32 MFMA (16 registers per lane each);
//   * slabs of A (and of B when it is stored N x K) sit in LDS as [row][k] with the row
//     stride padded by 4 floats, so one 16-byte LDS read gives a lane the operands of
//     four MFMA steps;  slabs of B stored K x N (or packed) sit as [k][n] and a lane
//     reads NB adjacent columns at once, which also makes its C stores NB floats wide;
//   * software pipeline, two LDS buffers, one barrier per slab: while slab t is being
//     multiplied, slab t+1 (fetched into registers one slab earlier) is written to the other
//     LDS buffer and slab t+2 is requested from global memory; operand fragments for the
//     next 8 columns of k are read from LDS while the current 8 are on the matrix pipe, and
//     the barrier sits before the last 8-column group so that the first fragments of the
//     next slab are already in flight when the current slab's last MFMAs issue.
//
// Lane maps of v_mfma_f32_32x32x2_f32 used below (lane l, l32 = l % 32, h = l / 32):
//   A operand: A[i = l32][k = h]      B operand: B[k = h][j = l32]
//   D register v: D[i = 8*(v/4) + 4*h + v%4][j = l32]
// The two k values of one MFMA step may be any two slab columns as long as A and B agree;
// step e of an 8-column group uses columns e (h = 0) and 4 + e (h = 1).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "fast_div.hpp"

namespace gemmf32 {

typedef float v2f __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
// Global-memory views with 4-byte alignment: operands whose base or leading dimension is not a
// multiple of 16 bytes are still moved with one 16-byte (or 8-byte) instruction per lane.
typedef v2f v2f_g __attribute__((aligned(4)));
typedef v4f v4f_g __attribute__((aligned(4)));

enum BMode : int { B_NN = 0, B_NT = 1, B_PACKED = 2 };
// A stored M x K (rows of k), or K x M (the transposed view of Section 6.3 applied to a): its slab
// then sits in LDS as [k][m] exactly like B stored K x N, a lane reads MB adjacent rows of the tile
// at once, and row r of MFMA block i is tile row MB*r + i.
enum AMode : int { A_MK = 0, A_KM = 1 };

constexpr int kPanel = 128;  // panel width P of the packed-B layout, in elements

// (fast_div.hpp: division of a walk position by a divisor that is fixed for the launch)
__device__ __forceinline__ int fast_div(int n, const FastDiv f)
{
    return f.magic == 0 ? n : (int)(__umulhi((unsigned)n, f.magic) >> f.shift);
}

struct KArgs {
    const float *A;
    const float *B;
    float *C;
    int M, N, K;
    int64_t lda, ldb, ldc;
    int64_t sA, sB, sC;      // batch strides in elements
    int tiles_m, tiles_n;    // tile grid of one product
    int group_m;             // tile rows per group in the tile walk
    int tiles_per_batch;     // tiles_m * tiles_n
    // divisions by tiles_per_batch, by group_m * tiles_n, by group_m and by the rows of the last, shorter group
    // (tiles_m % group_m, if any), see set_tile_walk
    FastDiv div_batch, div_group, div_rows, div_last_rows;
    int total_tiles;         // tiles_per_batch * batch == gridDim.x
    int n_padded;            // packed B: number of columns present in the buffer
    int k_total;             // split-K: length of the whole reduction (0: no split).  The "batch" index
                             // then counts K ranges of length K; the last one may be shorter
    int k_panel;             // packed B: rows per panel (the whole K, also when split)
    // Split tail: the tiles of the last, partly filled round (walk positions >= tail_first) are each
    // cut into tail_split K ranges of tail_k columns, so that the round occupies the whole chip; the
    // pieces go to dense BM x BN slots and tail_reduce_kernel sums them.  tail_split <= 1: off.
    int tail_first, tail_split, tail_k;
    float *tail_slots;
    // Or (quad != 0; tiles of at most 128 x 64): each tail tile is cut into its 32 x 32 blocks
    // (tail_split = their number) and a whole workgroup computes one block, its four waves sharing
    // every slab along k and adding up through LDS: a quarter of the tile's time, no second pass.
    int quad;
    // Strip: when N leaves at most kStripMax columns beyond whole tiles, the tiles cover columns [0, strip_n0)
    // (N above is strip_n0 then) and the strip_cols columns behind them are computed in the vector unit by
    // extra workgroups (ids >= strip_first; strip_r = 1, 2 or 4 rows per wave, four waves) that run beside
    // the tiles: a tile column of matrix work for a handful of columns would cost a whole round.
    // strip_cols == 0: off, and strip_first is the grid size.
    int strip_first, strip_cols, strip_n0, strip_r;
    int strip_wait;                 // pauses of 1024 cycles a strip workgroup takes before its first load
    // Epilogue: C = alpha * (A*B) + beta * C_old.  beta == 0: C_old is never read.  The paper's
    // product is alpha = 1, beta = 0.
    float alpha, beta;
#ifdef GEMMF32_TIMELINE
    unsigned long long *stamps;   // measurement build only: 8 slots per workgroup, see GEMMF32_STAMP
#endif
};

// Measurement build (-DGEMMF32_TIMELINE, a library of its own that bench.py --timeline loads): thread 0 of
// every workgroup writes the constant 100 MHz clock into slot i of its row of `stamps` as it passes:
//   0 kernel entry   1 first slab in LDS (before the first matrix instruction)   2 last whole slab multiplied
//   3 epilogue begins   4 (waves that share the slabs) sums in LDS   5 stores issued   6 hardware id
//   7 slabs 0 .. PF requested (between 0 and 1)
// (strip workgroups: 2 B's columns of the first chunk in LDS, 3 products summed over k, 5 sums over the lanes stored)
// The product library is built without the macro and contains none of this.
#ifdef GEMMF32_TIMELINE
constexpr int kTimelineMaxWorkgroups = 4096;
__device__ __forceinline__ void timeline_stamp(const KArgs &p, int i)
{
    if (p.stamps != nullptr && threadIdx.x == 0 && blockIdx.x < kTimelineMaxWorkgroups) p.stamps[blockIdx.x * 8 + i] = wall_clock64();
}
#define GEMMF32_STAMP(p, i) timeline_stamp(p, i)
#else
#define GEMMF32_STAMP(p, i) ((void)0)
#endif

template <int N> struct VecOf;
template <> struct VecOf<1> { typedef float type; typedef float gtype; };
template <> struct VecOf<2> { typedef v2f type; typedef v2f_g gtype; };
template <> struct VecOf<4> { typedef v4f type; typedef v4f_g gtype; };

template <int N> __device__ __forceinline__ float vget(const typename VecOf<N>::type &v, int i) { return v[i]; }
template <> __device__ __forceinline__ float vget<1>(const float &v, int) { return v; }

// WGK > 1: the waves of a workgroup also split every slab along k (wave w / (WGM*WGN) takes that
// share of the slab's 8-column groups) and their accumulators are added through LDS at the end: a
// 32 x 32 output block is then computed four times as fast as by one wave, with no second pass.
template <int BM_, int BN_, int BK_, int WGM_, int WGN_, int BMODE_, int OCC_ = 1, int PF_ = 1, int AMODE_ = A_MK,
          int WGK_ = 1>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_, WGK = WGK_;
    static constexpr int BMODE = BMODE_, OCC = OCC_, AMODE = AMODE_;
    static constexpr int PF = PF_;                             // slabs held in registers ahead of the LDS write
    static_assert(PF_ >= 1 && PF_ <= 4, "prefetch depth");
    static constexpr int THREADS = 64 * WGM * WGN * WGK;
    static constexpr int WM = BM / WGM, WN = BN / WGN;
    static constexpr int MB = WM / 32, NB = WN / 32;
    static constexpr int G = BK / 8;                           // 8-column groups per slab
    static constexpr int GQ = G / WGK;                         // of which one wave multiplies this many
    // Slabs with k contiguous ([row][k]: A stored M x K, B stored N x K): rows padded by 4 floats when a row
    // holds at least 32 columns of k (the 16-byte fragment reads of 8 consecutive rows and the 16-byte writes of
    // a row's 8 chunks then fall into distinct banks).  With 16 columns a padded row is 80 bytes and the writes
    // of four rows (4 chunks each) overlap in some banks (measured: 16.3 instead of 13.6 cycles per 16-byte
    // write instruction, a fifth of the kernel's LDS cycles spent in conflicts): those slabs are unpadded
    // instead and the 16-byte chunk c of row r sits at chunk position c ^ ((r / 4) % 4).  The LDS serves 16
    // lanes of a 16-byte access at a time from 64 banks: the writes of four rows are 256 contiguous bytes, and
    // 16 consecutive rows reading the same c hit 16 distinct 16-byte bank groups (measured 6.7 cycles per
    // read instruction, as for linear addresses; 16.3 without the XOR, 8.6 with (r / 2) % 4).
    static constexpr bool SWZ = (BK == 16);
    static constexpr int SA = (AMODE == A_KM) ? BM : (SWZ ? BK : BK + 4);   // A in LDS: [BM][SA], or [BK][BM] when stored K x M
    // B in LDS: [BN][SB] (NT) or [BK][SB] with SB >= BN; rows at least 64 floats apart keep the
    // fragment reads (one float from each of several rows) within reach of one address register
    static constexpr int SB = (BMODE == B_NT) ? (SWZ ? BK : BK + 4) : (BN < 64 ? 64 : BN);
    static constexpr int A_TILE = (AMODE == A_KM) ? BK * BM : BM * SA;
    static constexpr int B_TILE = (BMODE == B_NT) ? BN * SB : BK * SB;
    static constexpr int STAGE_FLOATS = A_TILE + B_TILE;
    static constexpr int LDS_BYTES = 2 * STAGE_FLOATS * 4;
    static constexpr int A_F4 = BM * BK / 4, A_ITERS = A_F4 / THREADS;
    static constexpr int B_F4 = BN * BK / 4, B_ITERS = B_F4 / THREADS;
    static constexpr int A_F4_ROW = (AMODE == A_KM) ? BM / 4 : BK / 4;    // 16-byte chunks per A row in the slab
    static constexpr int B_F4_ROW = (BMODE == B_NT) ? BK / 4 : BN / 4;    // per B row in the slab
    static_assert(BM % (32 * WGM) == 0 && BN % (32 * WGN) == 0, "wave tiles are multiples of 32");
    static_assert(BK % 16 == 0, "a slab holds an even number of 8-column groups");
    static_assert(A_F4 % THREADS == 0 && B_F4 % THREADS == 0, "loads divide evenly over threads");
    static_assert(NB == 1 || NB == 2 || NB == 4, "NB columns are read as one LDS vector");
    static_assert(AMODE == A_MK || MB == 1 || MB == 2 || MB == 4, "MB rows are read as one LDS vector");
    static_assert(AMODE == A_MK || BMODE != B_PACKED, "no packed B together with A stored K x M");
    static_assert(BMODE != B_PACKED || BN % kPanel == 0 || kPanel % BN == 0, "tile vs panel");
    static_assert(LDS_BYTES <= 160 * 1024, "fits the 160 KB of LDS per compute unit");
    static_assert(G % WGK == 0 && GQ >= 2 && GQ % 2 == 0, "every wave multiplies an even number of groups of a slab");
    static_assert(WGK == 1 || (WGM == 1 && WGN == 1), "k-split waves share the whole tile");
    static_assert(WGK == 1 || WGK * BM * (BN + 1) * 4 <= LDS_BYTES, "room for the final sum of the k-split accumulators");
};

// Maps the hardware workgroup id to a tile.  Workgroups are handed to the 8 XCDs round
// robin; ids are renumbered so that each XCD (own L2) receives one contiguous run of the
// tile walk, and the walk goes down `group_m` tile rows before moving one tile column so
// that a run forms a compact rectangle sharing rows of A and columns of B.
__device__ __forceinline__ int xcd_contiguous_id(int wg, int total)
{
    const int chunk = total >> 3, rem = total & 7;
    const int x = wg & 7, q = wg >> 3;
    return x * chunk + (x < rem ? x : rem) + q;
}
// position t of the tile walk of one product -> tile row / column
__device__ __forceinline__ void tile_coords(const KArgs &p, int t, int &tm, int &tn)
{
    const int gsz = p.group_m * p.tiles_n;
    const int grp = fast_div(t, p.div_group);
    const int first_m = grp * p.group_m;
    const bool last = p.tiles_m - first_m < p.group_m;
    const int gm = last ? (p.tiles_m - first_m) : p.group_m;
    const int r = t - grp * gsz;
    tn = last ? fast_div(r, p.div_last_rows) : fast_div(r, p.div_rows);
    tm = first_m + r - tn * gm;
}
// The tile grid of one product and the constants of its walk.
inline void set_tile_walk(KArgs &a, int tiles_m, int tiles_n, int group_m)
{
    a.tiles_m = tiles_m;
    a.tiles_n = tiles_n;
    a.tiles_per_batch = tiles_m * tiles_n;
    a.group_m = group_m;
    a.div_batch = make_fast_div((unsigned)a.tiles_per_batch);
    a.div_group = make_fast_div((unsigned)(group_m * tiles_n));
    a.div_rows = make_fast_div((unsigned)group_m);
    a.div_last_rows = make_fast_div((unsigned)(group_m > 0 ? tiles_m % group_m : 0));
}

// Barrier between LDS producers and consumers.  Only LDS traffic has to be complete: global
// loads requested for a later slab stay in flight across it.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N-1>{}).
template <class F, int... I> __device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Pins the issue order of the code that precedes it in the same basic block: N_MEM memory
// instructions (LDS reads, LDS writes, global loads, in program order) are spread evenly over
// N_MFMA MFMAs instead of being issued in a burst.  A burst from all waves of a workgroup at once
// fills the LDS queue, and the in-order wave then cannot issue its next MFMA.
template <int N_MFMA, int N_MEM> __device__ __forceinline__ void spread_memory_between_mfma()
{
    constexpr int MEM_MASK = 0x100 | 0x200 | 0x020;   // LDS read | LDS write | global load
    if constexpr (N_MEM == 0) {
        return;
    } else if constexpr (N_MEM <= N_MFMA) {
        constexpr int STRIDE = N_MFMA / N_MEM;
#pragma unroll
        for (int i = 0; i < N_MEM; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, STRIDE, 0);
            __builtin_amdgcn_sched_group_barrier(MEM_MASK, 1, 0);
        }
    } else {
        constexpr int Q = (N_MEM + N_MFMA - 1) / N_MFMA;
#pragma unroll
        for (int i = 0; i < N_MFMA; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(MEM_MASK, Q, 0);
        }
    }
}

__device__ __forceinline__ v4f load4(const float *src) { return *reinterpret_cast<const v4f_g *>(src); }

// A pointer that is the same in every lane, told to the compiler: it then lives in scalar registers.
__device__ __forceinline__ const float *uniform_pointer(const float *ptr)
{
    const unsigned long long u = reinterpret_cast<unsigned long long>(ptr);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)u), hi = __builtin_amdgcn_readfirstlane((unsigned)(u >> 32));
    return reinterpret_cast<const float *>(((unsigned long long)hi << 32) | lo);
}
// 16 bytes per lane from `origin` (uniform) + `byte_offset` (per lane, 32 bits) with buffer addressing:
// the origin travels in a scalar descriptor, so moving it from slab to slab is scalar arithmetic and
// the request needs no vector instruction to form its address.  (Between two matrix instructions of a
// wave a vector ALU instruction costs the matrix pipe 14 cycles or more and a load through a 64-bit
// per-lane address about 36; scalar instructions, LDS instructions and buffer loads cost next to nothing.)
// By default the range check of the descriptor is opened to the full 4 GB window; callers keep offsets below it.
// `bytes`: the descriptor's range; a request at or beyond it touches no memory and returns zeros.
__device__ __forceinline__ v4f buffer_load4(const float *origin, unsigned byte_offset, unsigned bytes = 0xFFFFFFFFu)
{
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(origin), 0, (int)bytes, 0x00020000 /* 32-bit data */);
    return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)byte_offset, 0, 0));
}

// One BM x BN tile.  EDGE = 0: every access is in range.  EDGE = 1: the tile crosses the M
// boundary (or, for B stored N x K / packed, the N boundary): whole 16-byte chunks are either in
// range or not.  EDGE = 2 (B stored K x N only): the tile crosses the N boundary, chunks of a
// row of B may be partly in range.  Out-of-range operands are loaded from a clamped (valid)
// address and replaced by zero with a select, so the steady-state loop stays branch free.
// EDGE = 3: the tile crosses a boundary of a matrix that is at least one tile long in that
// dimension: its origin is moved back so that it ends at the boundary, every load is in range as
// for EDGE = 0, and only the rows and columns the tile owns are stored (the others belong to its
// neighbour, which computes the same values).
// EDGE = 0 and 3 address the operands through buffer descriptors with 32-bit offsets from the tile's
// origin.  So does EDGE = 1 when A is stored M x K: rows past the end of a row-major operand lie past
// its last byte, so a descriptor whose range ends there masks them in hardware (zeros, no memory
// access, no select).  These need the tile's offsets to fit 32 bits; EDGE = 4 is EDGE = 1 with
// per-lane 64-bit pointers and selects, for any leading dimension (as are EDGE = 2, and EDGE = 1
// when A is stored K x M).
template <class T, int EDGE_MODE>
__device__ __forceinline__ void gemm_tile(const KArgs &p, float *lds, const int batch, const int tm, const int tn)
{
    constexpr bool SHIFTED = (EDGE_MODE == 3);
    constexpr int EDGE = SHIFTED ? 0 : (EDGE_MODE == 4 ? 1 : (EDGE_MODE == 5 ? 2 : EDGE_MODE));   // how the loads treat the boundaries
    constexpr bool RANGED = (EDGE_MODE == 1 && T::AMODE == A_MK);           // boundaries masked by the descriptors' ranges
    constexpr bool BUF = (EDGE == 0) || RANGED;                            // buffer addressing
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, G = T::G;
    constexpr int MB = T::MB, NB = T::NB, SA = T::SA, SB = T::SB;
    constexpr int NTHR = T::THREADS;
    constexpr int A_ITERS = T::A_ITERS, B_ITERS = T::B_ITERS;
    constexpr int A_F4_ROW = T::A_F4_ROW, B_F4_ROW = T::B_F4_ROW;
    constexpr bool B_KMAJOR = (T::BMODE == B_NT);           // B fragments are 4 consecutive k of one column
    constexpr int NBV = B_KMAJOR ? NB : 4;   // B fragment vectors per 8-column group
    // mode 5: as mode 2, for an N that is a multiple of 4: a 16-byte slot of B stored K x N then lies either
    // wholly inside a row or wholly beyond column N, so B is loaded 16 bytes at a time and masked per slot
    constexpr bool B_SLOTWISE = (T::BMODE == B_NN && EDGE_MODE == 5);
    constexpr bool B_ELEMENTWISE = (T::BMODE == B_NN && EDGE == 2 && !B_SLOTWISE);
    constexpr bool A_KMAJOR = (T::AMODE == A_MK);           // A fragments are 4 consecutive k of one row
    constexpr int NAV = A_KMAJOR ? MB : 4;                  // A fragment vectors per 8-column group
    constexpr bool A_ELEMENTWISE = (!A_KMAJOR && EDGE != 0);
    typedef typename VecOf<NB>::type vnb;
    typedef typename std::conditional<B_KMAJOR, v4f, vnb>::type bfrag_t;
    typedef typename VecOf<A_KMAJOR ? 4 : MB>::type afrag_t;

    const int m_own = tm * BM, n_own = tn * BN;               // first row / column this tile stores
    const int m0 = (SHIFTED && m_own + BM > p.M) ? p.M - BM : m_own;
    const int n0 = (SHIFTED && n_own + BN > p.N) ? p.N - BN : n_own;
    const float *__restrict__ A = p.A + (int64_t)batch * p.sA;
    const float *__restrict__ B = p.B + (int64_t)batch * p.sB;
    float *__restrict__ C = p.C + (int64_t)batch * p.sC;
    const int M = p.M, N = p.N;
    // split-K: this workgroup reduces over K range number `batch` (strides sA / sB step along k)
    const int K = (p.k_total > 0 && p.k_total - batch * p.K < p.K) ? (p.k_total - batch * p.K) : p.K;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int kq = wave / (T::WGM * T::WGN);                   // which share of every slab's groups (0 unless WGK > 1)
    const int wv = wave % (T::WGM * T::WGN);
    const int wm0 = (wv / T::WGN) * T::WM, wn0 = (wv % T::WGN) * T::WN;
    constexpr int GQ = T::GQ;

    // ---- per-thread load slots: global pointer (running: the next slab to request), LDS offset,
    // edge predicates ----
    const float *pa[A_ITERS];
    const float *pb[B_ITERS];
    int sa_off[A_ITERS], sb_off[B_ITERS];
    bool a_ok[A_ITERS];         // row of A in range (A stored K x M: first row of the chunk)
    int a_col[A_ITERS];         // A stored K x M: first tile row of the chunk (global index)
    int a_d[A_ITERS][4];        // A stored K x M at an edge: clamped offsets of the four elements
    bool b_ok[B_ITERS];         // NT: row of B in range; packed: chunk present; NN: first column in range
    int b_col[B_ITERS];         // NN / packed: first global column of the chunk
    int b_d[B_ITERS][4];        // NN, EDGE 2: clamped offsets of the four elements from pb[r]
    // slot r of a thread lies a fixed number of rows below its slot 0: the LDS addresses of all slots
    // are one register plus constants
    static_assert(NTHR % A_F4_ROW == 0 && NTHR % B_F4_ROW == 0, "slots of a thread share their column");
    static_assert(!T::SWZ || ((NTHR / 4) % 16 == 0), "slots of a thread share their swizzle");
    // (k-contiguous slabs of 16 columns: chunk position XORed with (row / 4) % 4, see Tile::SWZ)
    const int sa_base = (tid / A_F4_ROW) * SA +
                        ((T::SWZ && T::AMODE == A_MK) ? ((tid % A_F4_ROW) ^ (((tid / A_F4_ROW) >> 2) & 3)) : (tid % A_F4_ROW)) * 4;
    const int sb_base = (tid / B_F4_ROW) * SB +
                        ((T::SWZ && T::BMODE == B_NT) ? ((tid % B_F4_ROW) ^ (((tid / B_F4_ROW) >> 2) & 3)) : (tid % B_F4_ROW)) * 4;
#pragma unroll
    for (int r = 0; r < A_ITERS; ++r) {
        const int f = tid + r * NTHR;
        const int row = f / A_F4_ROW, c = (f % A_F4_ROW) * 4;
        sa_off[r] = sa_base + r * (NTHR / A_F4_ROW) * SA;
        if constexpr (A_KMAJOR) {
            a_ok[r] = (m0 + row < M);
            a_col[r] = 0;
            const int gi = (m0 + row < M) ? (m0 + row) : (M - 1);
            pa[r] = A + (int64_t)gi * p.lda + c;
        } else {
            const int gi = m0 + c;
            a_col[r] = gi;
            a_ok[r] = (gi < M);
            const int gic = (gi < M) ? gi : (M - 1);
            pa[r] = A + (int64_t)row * p.lda + gic;
#pragma unroll
            for (int e = 0; e < 4; ++e) a_d[r][e] = ((gi + e < M) ? (gi + e) : (M - 1)) - gic;
        }
    }
    auto a_slot_row = [&](int r) { return (tid + r * NTHR) / A_F4_ROW; };
    const int64_t a_step = A_KMAJOR ? BK : (int64_t)BK * p.lda;
    auto b_slot_row = [&](int r) {          // row of the B slab (k, or n for N x K storage) of slot r
        return (tid + r * NTHR) / B_F4_ROW;
    };
#pragma unroll
    for (int r = 0; r < B_ITERS; ++r) {
        const int f = tid + r * NTHR;
        const int row = b_slot_row(r), c = (f % B_F4_ROW) * 4;
        sb_off[r] = sb_base + r * (NTHR / B_F4_ROW) * SB;
        if constexpr (T::BMODE == B_NT) {
            b_ok[r] = (n0 + row < N);
            b_col[r] = 0;
            const int gj = (n0 + row < N) ? (n0 + row) : (N - 1);
            pb[r] = B + (int64_t)gj * p.ldb + c;
        } else if constexpr (T::BMODE == B_NN) {
            const int gj = n0 + c;
            b_col[r] = gj;
            b_ok[r] = (gj < N);
            const int gjc = (gj < N) ? gj : (B_SLOTWISE ? 0 : N - 1);   // slot-wise: the 16 bytes read stay inside the row
            pb[r] = B + (int64_t)row * p.ldb + gjc;
#pragma unroll
            for (int e = 0; e < 4; ++e) b_d[r][e] = ((gj + e < N) ? (gj + e) : (N - 1)) - gjc;
        } else {
            const int gj = n0 + c;
            b_col[r] = gj;
            b_ok[r] = (gj < p.n_padded);
            const int gjc = (gj < p.n_padded) ? gj : 0;
            pb[r] = B + ((int64_t)(gjc / kPanel) * p.k_panel + row) * kPanel + (gjc % kPanel);
        }
    }
    const int64_t b_step = (T::BMODE == B_NT) ? BK : (T::BMODE == B_NN ? (int64_t)BK * p.ldb : (int64_t)BK * kPanel);
    // BUF: the slots as 32-bit byte offsets from the tile's origin in each operand.  The origins are
    // uniform and, like the pointers of the other modes, stand at the next slab to request.
    // RANGED: end_a / end_b are one past the last element of the operand that this tile's K range may
    // read (last row, last column of the range); rows past the end start at or beyond them.
    unsigned va[A_ITERS], vb[B_ITERS];
    const float *org_a = nullptr, *org_b = nullptr, *end_a = nullptr, *end_b = nullptr;
    if constexpr (BUF) {
        org_a = uniform_pointer(A + (A_KMAJOR ? (int64_t)m0 * p.lda : (int64_t)m0));
        const int64_t b_origin = (T::BMODE == B_NT)   ? (int64_t)n0 * p.ldb
                                 : (T::BMODE == B_NN) ? (int64_t)n0
                                                      : (int64_t)(n0 / kPanel) * p.k_panel * kPanel + (n0 % kPanel);
        org_b = uniform_pointer(B + b_origin);
#pragma unroll
        for (int r = 0; r < A_ITERS; ++r) {
            const int f = tid + r * NTHR;
            va[r] = (unsigned)(((int64_t)(f / A_F4_ROW) * p.lda + (f % A_F4_ROW) * 4) * 4);
        }
#pragma unroll
        for (int r = 0; r < B_ITERS; ++r) {
            const int f = tid + r * NTHR;
            const int row = f / B_F4_ROW, c = (f % B_F4_ROW) * 4;
            if constexpr (T::BMODE == B_PACKED) {
                const int gj = n0 + c;
                vb[r] = (unsigned)((((int64_t)(gj / kPanel) * p.k_panel + row) * kPanel + (gj % kPanel) - b_origin) * 4);
            } else {
                vb[r] = (unsigned)(((int64_t)row * p.ldb + c) * 4);
            }
        }
        if constexpr (RANGED) {
            end_a = uniform_pointer(A + (int64_t)(M - 1) * p.lda + K);
            if constexpr (T::BMODE == B_NT) end_b = uniform_pointer(B + (int64_t)(N - 1) * p.ldb + K);
            else if constexpr (T::BMODE == B_PACKED)
                end_b = uniform_pointer(B + ((int64_t)(p.n_padded / kPanel - 1) * p.k_panel + K) * kPanel);
        }
    }
    // bytes from an origin to the end of its operand, as a descriptor range (the window is 4 GB at most)
    auto range_bytes = [&](const float *org, const float *end) {
        const uint64_t d = (uint64_t)((end - org) * 4);                  // never negative
        unsigned hi = (unsigned)(d >> 32);
        hi = __builtin_amdgcn_readfirstlane(hi);   // keeps the test on the high word: a 32-bit scalar compare (there is no
                                                   // scalar ordered compare of 64-bit values, and a vector one costs the matrix pipe)
        return hi != 0 ? 0xFFFFFFFFu : (unsigned)d;
    };
    // where slot r stands now, as a pointer (for the ragged last slab)
    auto a_slot_ptr = [&](int r) { return BUF ? org_a + (va[r] >> 2) : pa[r]; };
    auto b_slot_ptr = [&](int r) { return BUF ? org_b + (vb[r] >> 2) : pb[r]; };

    // Staging registers: PF sets.  Set s holds a slab between its global load and its LDS write.
    // One more set (index PF) carries slab 0 and is dead after the prologue.
    constexpr int PF = T::PF;
    v4f ra[PF + 1][A_ITERS], rb[PF + 1][B_ITERS];
    const v4f zero4 = {0.f, 0.f, 0.f, 0.f};

    // global -> registers for one load slot (slots 0..A_ITERS-1 are A, the rest B) of the slab its
    // pointer stands at (a whole slab, in range along k); the pointer then moves on by a_adv / b_adv
    // (one slab, or nothing once it stands at the last whole slab: later requests repeat that slab
    // and are never used).  The pointers live in registers of their own for the whole loop: an
    // address computed into a temporary per request ties the request to whatever else the
    // register allocator keeps in that temporary (fragments), and the in-order wave then waits on
    // chains of false dependencies.  Out-of-range rows and
    // columns come from a clamped address; they are zeroed when the slot is written to LDS
    // (masked_slot), not here, so that nothing has to wait for the load before then.
    auto load_slot = [&](auto slot_tag, auto set_tag, int64_t a_adv, int64_t b_adv) {
        constexpr int S = decltype(slot_tag)::value, SET = decltype(set_tag)::value;
        if constexpr (S < A_ITERS) {
            constexpr int r = S;
            v4f v;
            if constexpr (RANGED) {
                v = buffer_load4(org_a, va[r], range_bytes(org_a, end_a));
            } else if constexpr (BUF) {
                v = buffer_load4(org_a, va[r]);
            } else if constexpr (A_ELEMENTWISE) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = pa[r][a_d[r][e]];
            } else {
                v = load4(pa[r]);
            }
            ra[SET][r] = v;
            if constexpr (!BUF) pa[r] += a_adv;
        } else {
            constexpr int r = S - A_ITERS;
            v4f v;
            if constexpr (RANGED && T::BMODE != B_NN) {
                v = buffer_load4(org_b, vb[r], range_bytes(org_b, end_b));
            } else if constexpr (BUF) {
                v = buffer_load4(org_b, vb[r]);
            } else if constexpr (B_ELEMENTWISE) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = pb[r][b_d[r][e]];
            } else {
                v = load4(pb[r]);
            }
            rb[SET][r] = v;
            if constexpr (!BUF) pb[r] += b_adv;
            // the origins move once per slab, after the last slot's request
            if constexpr (BUF && r == B_ITERS - 1) { org_a += a_adv; org_b += b_adv; }
        }
    };
    auto masked_slot = [&](auto slot_tag, v4f v) {
        constexpr int S = decltype(slot_tag)::value;
        if constexpr (EDGE != 0 && !BUF) {
            if constexpr (S < A_ITERS) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool ok = A_ELEMENTWISE ? (a_col[S] + e < M) : a_ok[S];
                    v[e] = ok ? v[e] : 0.f;
                }
            } else if constexpr (B_ELEMENTWISE || B_SLOTWISE || T::BMODE != B_NN) {
                constexpr int r = S - A_ITERS;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool ok = B_ELEMENTWISE ? (b_col[r] + e < N) : b_ok[r];
                    v[e] = ok ? v[e] : 0.f;
                }
            }
        }
        return v;
    };
    // requests the slab the pointers stand at; `advance`: a later whole slab exists
    auto load_slab = [&](auto set_tag, bool advance) {
        const int64_t a_adv = advance ? a_step : 0, b_adv = advance ? b_step : 0;
        static_for<A_ITERS + B_ITERS>([&](auto slot_tag) { load_slot(slot_tag, set_tag, a_adv, b_adv); });
    };

    // ---- the first requests go out before the rest of the set-up -----------------------------------
    // A workgroup is alone on its SIMDs at this point and executes its set-up (fragment offsets, the
    // accumulators' zeros, the epilogue's constants: some hundred instructions, one after the other)
    // at about eight cycles each; with the requests first, that time runs under the memory latency.
    const int nkf = __builtin_amdgcn_readfirstlane(K / BK);   // uniform; kept in a scalar register (see gemm_kernel)
    const int kleft = K - nkf * BK;
    typedef std::integral_constant<int, PF> first_set;
    // Late start.  Requesting slabs 0 .. PF before anything else keeps the workgroup's way to memory busy with
    // slabs 1 .. PF (a compute unit takes in 64 bytes per cycle: 0.2 us per 32 KB slab) while slab 0, the only
    // one the first matrix instruction waits for, queues with them: measured, a 64 x 64 x 64 tile issued its
    // requests for 1.06 us and had slab 0 in LDS 0.24 us later.  Tiles with slabs of at least four 8-column groups
    // and two slabs in registers request slab 0 alone and leave slabs 1 .. PF to the first half of slab 0's
    // own matrix work (slab_body with FIRST), where their way to memory is idle anyway.
    constexpr bool LATE_START = (T::GQ >= 4 && PF >= 2);
    [[maybe_unused]] v4f ta[A_ITERS], tb[B_ITERS];
    if (nkf > 0) {
        const int last = nkf - 1;
        // A ragged K: the K % BK odd columns come first, the whole slabs after them.  Their loads are
        // requested ahead of slabs 0 .. PF, they pass through LDS buffer 1 and are multiplied while
        // slab 0 is still on its way, so that the ragged part costs one barrier instead of a load
        // latency of its own at the end.  Every slot is one 16-byte load from a position that lies inside
        // the operand (columns at or beyond kleft re-read column 0, rows re-read row 0; K >= kleft + BK
        // here, so the 16 bytes never reach past column K); what lies at or beyond kleft is zeroed in
        // both operands before it reaches LDS.
        if (kleft > 0) {
            static_for<A_ITERS>([&](auto r_tag) {
                constexpr int r = decltype(r_tag)::value;
                const int f = tid + r * NTHR;
                // k index of the slot's first element, and how far back (in elements) the load moves
                const int k0 = A_KMAJOR ? (f % A_F4_ROW) * 4 : f / A_F4_ROW;
                const int64_t back = (k0 < kleft) ? 0 : (A_KMAJOR ? (int64_t)k0 : (int64_t)k0 * p.lda);
                v4f v;
                if constexpr (RANGED) v = buffer_load4(org_a, va[r] - (unsigned)(back * 4), range_bytes(org_a, end_a));
                else if constexpr (BUF) v = buffer_load4(org_a, va[r] - (unsigned)(back * 4));
                else if constexpr (A_ELEMENTWISE) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (pa[r] - back)[a_d[r][e]];
                } else v = load4(pa[r] - back);
                ta[r] = v;
            });
            static_for<B_ITERS>([&](auto r_tag) {
                constexpr int r = decltype(r_tag)::value;
                const int f = tid + r * NTHR;
                const int k0 = B_KMAJOR ? (f % B_F4_ROW) * 4 : f / B_F4_ROW;
                const int64_t kstride = (T::BMODE == B_NT) ? 1 : (T::BMODE == B_NN ? p.ldb : (int64_t)kPanel);
                const int64_t back = (k0 < kleft) ? 0 : (int64_t)k0 * kstride;
                v4f v;
                if constexpr (RANGED && T::BMODE != B_NN) v = buffer_load4(org_b, vb[r] - (unsigned)(back * 4), range_bytes(org_b, end_b));
                else if constexpr (BUF) v = buffer_load4(org_b, vb[r] - (unsigned)(back * 4));
                else if constexpr (B_ELEMENTWISE) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (pb[r] - back)[b_d[r][e]];
                } else v = load4(pb[r] - back);
                tb[r] = v;
            });
            // the whole slabs start kleft columns further along k
            const int64_t a_skip = A_KMAJOR ? (int64_t)kleft : (int64_t)kleft * p.lda;
            const int64_t b_skip = (T::BMODE == B_NT) ? (int64_t)kleft : (T::BMODE == B_NN ? (int64_t)kleft * p.ldb : (int64_t)kleft * kPanel);
            if constexpr (BUF) {
                org_a = uniform_pointer(org_a + a_skip);
                org_b = uniform_pointer(org_b + b_skip);
            } else {
#pragma unroll
                for (int r = 0; r < A_ITERS; ++r) pa[r] += a_skip;
#pragma unroll
                for (int r = 0; r < B_ITERS; ++r) pb[r] += b_skip;
            }
        }
        // slabs 0 .. PF are all requested before the first of them is waited for: slab 0 into the
        // extra register set, slab j (1 <= j <= PF) into set j % PF, where the loop expects it
        load_slab(first_set{}, 0 < last);                       // slab 0; the pointers move to slab min(1, last)
        // (late start, see slab_body: with more than PF slabs the loop's first round requests slabs 1 .. PF itself)
        if (!(LATE_START && nkf > PF)) {
            static_for<PF>([&](auto j_tag) {
                constexpr int j = decltype(j_tag)::value + 1;   // slab min(j, last); then on to min(j + 1, last)
                load_slab(std::integral_constant<int, j % PF>{}, j < last);
            });
        }
        GEMMF32_STAMP(p, 7);
    }
    // global -> registers (set 0) for the ragged last slab: kleft (< BK) columns of k remain.  After
    // the main loop the pointers stand at the last whole slab (at slab 0 if there is none).
    auto load_tail = [&](bool after_whole_slabs, int kleft) {
        const int64_t a_off = after_whole_slabs ? a_step : 0, b_off = after_whole_slabs ? b_step : 0;
#pragma unroll
        for (int r = 0; r < A_ITERS; ++r) {
            const int c = ((tid + r * NTHR) % A_F4_ROW) * 4;
            v4f v = zero4;
            if constexpr (A_KMAJOR) {
                if (a_ok[r]) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (c + e < kleft) v[e] = (a_slot_ptr(r) + a_off)[e];
                }
            } else {
                if (a_slot_row(r) < kleft && a_ok[r]) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (a_col[r] + e < M) v[e] = (a_slot_ptr(r) + a_off)[e];   // the slot's pointer is unclamped when a_ok
                }
            }
            ra[0][r] = v;
        }
#pragma unroll
        for (int r = 0; r < B_ITERS; ++r) {
            const float *src = b_slot_ptr(r) + b_off;
            v4f v = zero4;
            if constexpr (T::BMODE == B_NT) {
                const int c = ((tid + r * NTHR) % B_F4_ROW) * 4;
                if (b_ok[r]) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (c + e < kleft) v[e] = src[e];
                }
            } else if constexpr (T::BMODE == B_NN) {
                if (b_slot_row(r) < kleft && b_ok[r]) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (b_col[r] + e < N) v[e] = src[e];   // pb[r] is unclamped when b_ok
                }
            } else {
                if (b_slot_row(r) < kleft && b_ok[r]) v = load4(src);
            }
            rb[0][r] = v;
        }
    };
    auto store_slab = [&](int stage, auto set_tag) {
        constexpr int SET = decltype(set_tag)::value;
        float *As = lds + stage * T::STAGE_FLOATS;
        float *Bs = As + T::A_TILE;
        static_for<A_ITERS>([&](auto r_tag) {
            constexpr int r = decltype(r_tag)::value;
            *reinterpret_cast<v4f *>(&As[sa_off[r]]) = masked_slot(r_tag, ra[SET][r]);
        });
        static_for<B_ITERS>([&](auto r_tag) {
            constexpr int r = decltype(r_tag)::value;
            *reinterpret_cast<v4f *>(&Bs[sb_off[r]]) = masked_slot(std::integral_constant<int, A_ITERS + r>{}, rb[SET][r]);
        });
    };
    // Moving a staged slab into LDS and requesting a later slab into the same registers is a list of
    // actions executed in order, one per slot: write the slot to LDS, reload it.
    constexpr int N_ACTIONS = A_ITERS + B_ITERS;
    auto do_action = [&](auto a_tag, int stage, auto set_tag, int64_t a_adv, int64_t b_adv) {
        constexpr int a = decltype(a_tag)::value, SET = decltype(set_tag)::value;
        float *As = lds + stage * T::STAGE_FLOATS;
        if constexpr (a < A_ITERS) *reinterpret_cast<v4f *>(&As[sa_off[a]]) = masked_slot(a_tag, ra[SET][a]);
        else *reinterpret_cast<v4f *>(&As[T::A_TILE + sb_off[a - A_ITERS]]) = masked_slot(a_tag, rb[SET][a - A_ITERS]);
        load_slot(a_tag, set_tag, a_adv, b_adv);
    };

    // ---- LDS -> fragments -> MFMA -----------------------------------------------------------
    struct Frag {
        afrag_t a[NAV];
        bfrag_t b[NBV];
    };
    // (group g of this wave is group kq * GQ + g of the slab)
    // k-contiguous slabs: the lane's row, and where the 16 bytes of group g lie in it (columns 8g + 4 * half ..;
    // swizzled slabs: chunk 2g + half at position (2g + half) ^ ((row / 4) % 4), one offset per group)
    const int a_frag_off = (A_KMAJOR ? ((wm0 + l32) * SA + (T::SWZ ? 0 : 4 * half)) : (4 * half * SA + wm0 + MB * l32)) +
                           8 * GQ * kq * (A_KMAJOR ? 1 : SA);
    const int b_frag_off = ((T::BMODE == B_NT) ? (T::A_TILE + (wn0 + l32) * SB + (T::SWZ ? 0 : 4 * half))
                                               : (T::A_TILE + 4 * half * SB + wn0 + NB * l32)) +
                           8 * GQ * kq * (T::BMODE == B_NT ? 1 : SB);
    int k_off[G];                                     // offset of group g's 16 bytes within a k-contiguous row
#pragma unroll
    for (int g = 0; g < G; ++g) k_off[g] = T::SWZ ? 4 * ((2 * g + half) ^ ((l32 >> 2) & 3)) : 8 * g;
    auto read_frag = [&](Frag &fr, int stage, int g) {
        const float *base = lds + stage * T::STAGE_FLOATS;
        if constexpr (A_KMAJOR) {
#pragma unroll
            for (int i = 0; i < MB; ++i)   // row of block i: wm0 + 32*i + l32
                fr.a[i] = *reinterpret_cast<const v4f *>(base + a_frag_off + 32 * i * SA + k_off[g]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)    // row of block i: wm0 + MB*l32 + i
                fr.a[e] = *reinterpret_cast<const afrag_t *>(base + a_frag_off + (8 * g + e) * SA);
        }
        if constexpr (T::BMODE == B_NT) {
#pragma unroll
            for (int j = 0; j < NB; ++j)   // column of block j: wn0 + 32*j + l32
                fr.b[j] = *reinterpret_cast<const v4f *>(base + b_frag_off + 32 * j * SB + k_off[g]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)    // column of block j: wn0 + NB*l32 + j
                fr.b[e] = *reinterpret_cast<const vnb *>(base + b_frag_off + (8 * g + e) * SB);
        }
    };

    v16f acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    auto mfma_group = [&](const Frag &fr) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    float av, bv;
                    if constexpr (A_KMAJOR) av = fr.a[i][e];
                    else av = vget<MB>(fr.a[e], i);
                    if constexpr (B_KMAJOR) bv = fr.b[j][e];
                    else bv = vget<NB>(fr.b[e], j);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i][j], 0, 0, 0);
                }
    };

    // ---- main loop over the full slabs --------------------------------------------------------
    // Issue order inside a slab is pinned with scheduling groups: the LDS reads, LDS writes and
    // global loads are spread one at a time between MFMAs instead of being issued in a burst
    // (a burst from all waves at once fills the LDS queue and stalls MFMA issue behind it).
    Frag f0, f1;
    constexpr int N_MFMA = 4 * MB * NB;            // MFMAs of one 8-column group
    constexpr int N_READ = NAV + NBV;              // LDS reads of one fragment set
    // The actions of a slab run in the groups that precede the barrier (all but the last one),
    // the same number in each, in order.
    constexpr int MOVE_GROUPS = GQ - 1;
    // Slab t: multiply it out of LDS buffer t % 2 while
    // slab t+1 goes from register set (t+1) % PF into the other buffer and slab t+1+PF is requested
    // into the same registers (past the end: a harmless re-request of the last full slab).
    auto slab_body = [&](const int t, auto par_tag, auto more_tag, auto first_tag) {
        constexpr int PAR = decltype(par_tag)::value;      // t % PF (register set choice)
        constexpr bool MORE = decltype(more_tag)::value;
        // the first slab of a late start: slabs 1 .. PF are requested in its first half (slab j into set j % PF,
        // slab 1's slots first), the actions follow in its second half, when slab 1 has had time to arrive
        constexpr bool FIRST = decltype(first_tag)::value;
        static_assert(!FIRST || (MORE && PAR == 0), "the first slab of more than PF");
        const int cur = t & 1;
        typedef std::integral_constant<int, (PAR + 1) % PF> set_t;
        // this slab requests slab min(t + 1 + PF, nkf - 1); the pointers move on if the next request is a later one
        const bool advance = (t + 2 + PF < nkf);
        const int64_t a_adv = advance ? a_step : 0, b_adv = advance ? b_step : 0;
        static_for<GQ>([&](auto g_tag) {
            constexpr int g = decltype(g_tag)::value;
            Frag &now = (g & 1) ? f1 : f0;
            Frag &next = (g & 1) ? f0 : f1;
            constexpr bool READS = (g + 1 < GQ) || MORE;
            if constexpr (g + 1 < GQ) {
                read_frag(next, cur, g + 1);
            } else if constexpr (MORE) {
                lds_barrier();                 // slab t+1 is complete in the other buffer
                read_frag(next, cur ^ 1, 0);
            }
            // early requests of a first slab: request e is slot e % N_ACTIONS of slab 1 + e / N_ACTIONS
            constexpr int EARLY_GROUPS = FIRST ? GQ / 2 : 0;
            constexpr int N_EARLY = PF * N_ACTIONS;
            constexpr int E_FIRST = (g < EARLY_GROUPS) ? (g * N_EARLY + EARLY_GROUPS - 1) / (EARLY_GROUPS > 0 ? EARLY_GROUPS : 1) : 0;
            constexpr int E_END = (g < EARLY_GROUPS) ? ((g + 1) * N_EARLY + EARLY_GROUPS - 1) / (EARLY_GROUPS > 0 ? EARLY_GROUPS : 1) : 0;
            if constexpr (E_END > E_FIRST) {
                static_for<E_END - E_FIRST>([&](auto i_tag) {
                    constexpr int e = E_FIRST + decltype(i_tag)::value;
                    constexpr int j = 1 + e / N_ACTIONS;            // slab min(j, nkf - 1); then on to min(j + 1, nkf - 1)
                    const bool on = (j < nkf - 1);
                    load_slot(std::integral_constant<int, e % N_ACTIONS>{}, std::integral_constant<int, j % PF>{},
                              on ? a_step : 0, on ? b_step : 0);
                });
            }
            // action i runs in group i * (groups with actions) / N_ACTIONS: spread as evenly as the counts allow
            // over the groups that precede the barrier (a first slab: over the later ones of them)
            constexpr int A_GROUPS = MOVE_GROUPS - EARLY_GROUPS;
            constexpr int ga = g - EARLY_GROUPS;
            constexpr int A_FIRST = (ga >= 0 && ga < A_GROUPS) ? (ga * N_ACTIONS + A_GROUPS - 1) / A_GROUPS : 0;
            constexpr int A_END = (ga >= 0 && ga < A_GROUPS) ? ((ga + 1) * N_ACTIONS + A_GROUPS - 1) / A_GROUPS : 0;
            constexpr int COUNT = MORE ? A_END - A_FIRST : 0;
            constexpr int MOVE_MEM = 2 * COUNT + (E_END - E_FIRST);    // one LDS write and one global load per action
            if constexpr (COUNT > 0) {
                static_for<COUNT>([&](auto i_tag) {
                    do_action(std::integral_constant<int, A_FIRST + decltype(i_tag)::value>{}, cur ^ 1, set_t{}, a_adv, b_adv);
                });
            }
            mfma_group(now);
            spread_memory_between_mfma<N_MFMA, (READS ? N_READ : 0) + MOVE_MEM>();
        });
    };
    typedef std::integral_constant<int, 0> i0;
    typedef std::integral_constant<int, 1> i1;
    if (nkf > 0) {
        if (kleft > 0) {
            float *As = lds + T::STAGE_FLOATS, *Bs = As + T::A_TILE;          // buffer 1
            static_for<A_ITERS>([&](auto r_tag) {
                constexpr int r = decltype(r_tag)::value;
                const int f = tid + r * NTHR;
                const int k0 = A_KMAJOR ? (f % A_F4_ROW) * 4 : f / A_F4_ROW;
                v4f v = masked_slot(r_tag, ta[r]);
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = ((A_KMAJOR ? k0 + e : k0) < kleft) ? v[e] : 0.f;
                *reinterpret_cast<v4f *>(&As[sa_off[r]]) = v;
            });
            static_for<B_ITERS>([&](auto r_tag) {
                constexpr int r = decltype(r_tag)::value;
                const int f = tid + r * NTHR;
                const int k0 = B_KMAJOR ? (f % B_F4_ROW) * 4 : f / B_F4_ROW;
                v4f v = masked_slot(std::integral_constant<int, A_ITERS + r>{}, tb[r]);
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = ((B_KMAJOR ? k0 + e : k0) < kleft) ? v[e] : 0.f;
                *reinterpret_cast<v4f *>(&Bs[sb_off[r]]) = v;
            });
            lds_barrier();
            // (the fragments of a group are read while the group before it is multiplied)
            if (8 * GQ * kq < kleft) read_frag(f0, 1, 0);
            static_for<GQ>([&](auto g_tag) {
                constexpr int g = decltype(g_tag)::value;
                if (8 * (GQ * kq + g) < kleft) {
                    Frag &now = (g & 1) ? f1 : f0;
                    if constexpr (g + 1 < GQ) {
                        if (8 * (GQ * kq + g + 1) < kleft) read_frag((g & 1) ? f0 : f1, 1, g + 1);
                    }
                    mfma_group(now);
                }
            });
        }
        store_slab(0, first_set{});
        lds_barrier();
        GEMMF32_STAMP(p, 1);
        read_frag(f0, 0, 0);
        // the loop is unrolled PF times so that the register set of every slab is a compile-time choice
        int t = 0;
        if constexpr (LATE_START) {
            if (PF < nkf) {
                static_for<PF>([&](auto i_tag) {
                    slab_body(decltype(i_tag)::value, i_tag, std::true_type{}, std::integral_constant<bool, decltype(i_tag)::value == 0>{});
                });
                t = PF;
            }
        }
        for (; t + PF < nkf; t += PF)
            static_for<PF>([&](auto i_tag) { slab_body(t + decltype(i_tag)::value, i_tag, std::true_type{}, std::false_type{}); });
        const int rest = nkf - t;                  // 1 .. PF slabs left; the last one requests nothing
        static_for<PF>([&](auto i_tag) {
            constexpr int i = decltype(i_tag)::value;
            if constexpr (i + 1 < PF) {
                if (i + 1 < rest) slab_body(t + i, i_tag, std::true_type{}, std::false_type{});
                else if (i + 1 == rest) slab_body(t + i, i_tag, std::false_type{}, std::false_type{});
            } else {
                if (PF == 1 || i + 1 == rest) slab_body(t + i, i_tag, std::false_type{}, std::false_type{});
            }
        });
    }
    GEMMF32_STAMP(p, 2);
    // ---- a K shorter than one slab: its K % BK columns, not pipelined ----------------------------
    if (kleft > 0 && nkf == 0) {
        load_tail(false, kleft);
        __syncthreads();                           // everyone is done reading both buffers
        store_slab(0, i0{});
        __syncthreads();
#pragma unroll
        for (int g = 0; g < GQ; ++g) {
            if (8 * (GQ * kq + g) < kleft) {
                read_frag(f0, 0, g);
                mfma_group(f0);
            }
        }
    }

    GEMMF32_STAMP(p, 3);
    // ---- epilogue: accumulators -> C (overwrite; predicated at the M / N edges) ---------------
    auto row_ok = [&](int gi) { return SHIFTED ? gi >= m_own : (EDGE == 0 || gi < M); };
    auto cols_ok = [&](int gj, int n) { return SHIFTED ? gj >= n_own : (EDGE == 0 || gj + n <= N); };
    const float alpha = p.alpha, beta = p.beta;
    const bool add_old = (beta != 0.f);                      // uniform over the grid
    // Tiles addressed through 32-bit offsets (BUF) store the same way: through a buffer descriptor based
    // at the tile's origin in C, with the row's byte offset (a compile-time row number times ldc) in a
    // scalar register and one 32-bit byte offset per lane, computed once.  A store then needs no vector
    // address arithmetic; 64-bit per-lane products for every element took about as long as the stores
    // themselves.  run_tile sends a tile here only if (BM - 1) * ldc + BN fits 30 bits.
    [[maybe_unused]] __amdgpu_buffer_rsrc_t c_rsrc;
    if constexpr (BUF)
        c_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(uniform_pointer(C + (int64_t)m0 * p.ldc + n0)), 0, -1,
                                                   0x00020000);
    [[maybe_unused]] const int ldc32 = __builtin_amdgcn_readfirstlane((int)p.ldc);   // uniform; said so, as the row offsets below must be scalar
    // element(s) at row `crow` (uniform), lane byte offset `off`: C = alpha * value (+ beta * C_old)
    auto put = [&](auto old_tag, int crow, unsigned off, auto value) {
        typedef decltype(value) V;
        constexpr bool ADD_OLD = decltype(old_tag)::value;
        const int row_bytes = crow * ldc32 * 4;
        V o = alpha * value;
        if constexpr (std::is_same<V, float>::value) {
            if constexpr (ADD_OLD) o += beta * __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(c_rsrc, (int)off, row_bytes, 0));
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, o), c_rsrc, (int)off, row_bytes, 0);
        } else if constexpr (sizeof(V) == 8) {
            typedef unsigned u2 __attribute__((ext_vector_type(2)));
            if constexpr (ADD_OLD) o += beta * __builtin_bit_cast(V, __builtin_amdgcn_raw_buffer_load_b64(c_rsrc, (int)off, row_bytes, 0));
            __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u2, o), c_rsrc, (int)off, row_bytes, 0);
        } else {
            typedef unsigned u4 __attribute__((ext_vector_type(4)));
            if constexpr (ADD_OLD) o += beta * __builtin_bit_cast(V, __builtin_amdgcn_raw_buffer_load_b128(c_rsrc, (int)off, row_bytes, 0));
            // A 16-byte store takes the row offset in its vector offset.  With the row offset in the scalar
            // offset the compiler leaves no wait state between the store and the next write of its four data
            // registers (that form is documented as needing none; with a constant scalar offset it inserts them),
            // and the lanes read last then stored the next row's value in their fourth dword: seen with
            // 128 x 256 tiles, two workgroups to a compute unit, in results that changed from run to run.
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, o), c_rsrc, (int)off + row_bytes, 0, 0);
        }
    };
    if constexpr (T::WGK > 1) {
        // the waves hold partial sums of the same tile: through LDS (element (r, c) of wave w at
        // red[w][r * (BN + 1) + c]), added in wave order, stored by all threads
        __syncthreads();                                      // the slab buffers are free
        float *red = lds;
        constexpr int RS = BN + 1, RW = BM * RS;
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int mrow = 8 * (v / 4) + 4 * half + (v % 4);
                    const int r = A_KMAJOR ? 32 * i + mrow : MB * mrow + i;
                    const int c = (T::BMODE == B_NT) ? 32 * j + l32 : NB * l32 + j;
                    red[kq * RW + r * RS + c] = acc[i][j][v];
                }
        __syncthreads();
        GEMMF32_STAMP(p, 4);
        constexpr int PASS_ROWS = NTHR / BN;                  // rows one pass of all threads covers
        const int li = tid / BN, lj = tid % BN;
        if constexpr (BUF) {
            const unsigned off = (unsigned)(li * ldc32 + lj) * 4u;
            const int row_lo = SHIFTED ? m_own - m0 - li : 0;                 // this lane stores rows crow in [row_lo, row_hi)
            const int row_hi = (EDGE != 0) ? M - m0 - li : BM;
            const bool col_ok = cols_ok(n0 + lj, 1);
            auto pass = [&](auto old_tag) {
#pragma unroll
                for (int t = 0; t < BM / PASS_ROWS; ++t) {
                    const int crow = PASS_ROWS * t;
                    float sum = red[(li + crow) * RS + lj];
#pragma unroll
                    for (int w = 1; w < T::WGK; ++w) sum += red[w * RW + (li + crow) * RS + lj];
                    if (col_ok && crow >= row_lo && crow < row_hi) put(old_tag, crow, off, sum);
                }
            };
            if (add_old) pass(std::true_type{});
            else pass(std::false_type{});
            return;
        }
#pragma unroll
        for (int t = 0; t < BM * BN / NTHR; ++t) {
            const int i = li + PASS_ROWS * t, j = lj;
            const int gi = m0 + i, gj = n0 + j;
            float sum = red[i * RS + j];
#pragma unroll
            for (int w = 1; w < T::WGK; ++w) sum += red[w * RW + i * RS + j];
            if (row_ok(gi) && cols_ok(gj, 1)) {
                float *dst = C + (int64_t)gi * p.ldc + gj;
                float r = alpha * sum;
                if (add_old) r += beta * *dst;
                *dst = r;
            }
        }
        return;
    }
    if constexpr (BUF) {
        const int lane_row = wm0 + (A_KMAJOR ? 4 : 4 * MB) * half;
        const int lane_col = wn0 + (T::BMODE == B_NT ? l32 : NB * l32);
        const unsigned off = (unsigned)(lane_row * ldc32 + lane_col) * 4u;
        const int row_lo = SHIFTED ? m_own - m0 - lane_row : 0;                // rows crow in [row_lo, row_hi) are this lane's to store
        const int row_hi = (EDGE != 0) ? M - m0 - lane_row : BM;
        bool col_ok[NB], all_cols = true;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            col_ok[j] = cols_ok(n0 + lane_col + (T::BMODE == B_NT ? 32 * j : j), 1);
            all_cols = all_cols && col_ok[j];
        }
        auto pass = [&](auto old_tag) {
#pragma unroll
            for (int i = 0; i < MB; ++i) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int crow = A_KMAJOR ? 32 * i + 8 * (v / 4) + (v % 4) : MB * (8 * (v / 4) + (v % 4)) + i;
                    const bool rok = crow >= row_lo && crow < row_hi;
                    if constexpr (T::BMODE == B_NT) {
#pragma unroll
                        for (int j = 0; j < NB; ++j)
                            if (rok && col_ok[j]) put(old_tag, crow, off + 128u * j, acc[i][j][v]);
                    } else {
                        bool done = false;
                        if constexpr (NB > 1) {
                            if (rok && all_cols) {
                                vnb o;
#pragma unroll
                                for (int j = 0; j < NB; ++j) o[j] = acc[i][j][v];
                                put(old_tag, crow, off, o);
                                done = true;
                            }
                        }
                        if (!done) {
#pragma unroll
                            for (int j = 0; j < NB; ++j)
                                if (rok && col_ok[j]) put(old_tag, crow, off + 4u * j, acc[i][j][v]);
                        }
                    }
                }
            }
        };
        if (add_old) pass(std::true_type{});
        else pass(std::false_type{});
        return;
    }
#pragma unroll
    for (int i = 0; i < MB; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int mrow = 8 * (v / 4) + 4 * half + (v % 4);          // row of the MFMA block
            const int gi = m0 + wm0 + (A_KMAJOR ? 32 * i + mrow : MB * mrow + i);
            if constexpr (T::BMODE == B_NT) {
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const int gj = n0 + wn0 + 32 * j + l32;
                    if (row_ok(gi) && cols_ok(gj, 1)) {
                        float *dst = C + (int64_t)gi * p.ldc + gj;
                        float r = alpha * acc[i][j][v];
                        if (add_old) r += beta * *dst;
                        *dst = r;
                    }
                }
            } else {
                const int gj = n0 + wn0 + NB * l32;
                float *dst = C + (int64_t)gi * p.ldc + gj;
                bool done = false;
                if constexpr (NB > 1) {
                    if (row_ok(gi) && cols_ok(gj, NB)) {
                        typedef typename VecOf<NB>::gtype gvec;
                        vnb o;
#pragma unroll
                        for (int j = 0; j < NB; ++j) o[j] = alpha * acc[i][j][v];
                        if (add_old) {
                            const vnb old = *reinterpret_cast<const gvec *>(dst);
                            o += beta * old;
                        }
                        *reinterpret_cast<gvec *>(dst) = o;
                        done = true;
                    }
                }
                if (!done) {
#pragma unroll
                    for (int j = 0; j < NB; ++j)
                        if (row_ok(gi) && cols_ok(gj + j, 1)) {
                            float r = alpha * acc[i][j][v];
                            if (add_old) r += beta * dst[j];
                            dst[j] = r;
                        }
                }
            }
        }
    }
}

// One tile of shape T at tile coordinates (tm, tn): picks how its boundaries are treated.
template <class T>
__device__ __forceinline__ void run_tile(const KArgs &q, float *lds, int batch, int tm, int tn)
{
    // The tile's coordinates are the same in every lane; said explicitly, because they come out of
    // integer divisions (done in the vector unit), and everything derived from them -- origins,
    // slab counts, buffer descriptors -- has to stay in scalar registers.
    batch = __builtin_amdgcn_readfirstlane(batch);
    tm = __builtin_amdgcn_readfirstlane(tm);
    tn = __builtin_amdgcn_readfirstlane(tn);
    const bool m_edge = (tm + 1) * T::BM > q.M, n_edge = (tn + 1) * T::BN > q.N;
    // the in-range paths address a tile with 32-bit byte offsets from its origin
    constexpr int64_t kSpanLimit = (1LL << 30) - 64;                       // elements: 4 GB less a margin
    const int64_t a_span = (T::AMODE == A_MK) ? (int64_t)(T::BM - 1) * q.lda + T::BK : (int64_t)(T::BK - 1) * q.lda + T::BM;
    const int64_t b_span = (T::BMODE == B_NT)   ? (int64_t)(T::BN - 1) * q.ldb + T::BK
                           : (T::BMODE == B_NN) ? (int64_t)(T::BK - 1) * q.ldb + T::BN
                                                : ((int64_t)((T::BN + kPanel - 1) / kPanel) * q.k_panel + T::BK) * kPanel;
    const int64_t c_span = (int64_t)(T::BM - 1) * q.ldc + T::BN;            // the epilogue of these paths: 32-bit offsets into C too
    const bool offsets_fit_32 = a_span < kSpanLimit && b_span < kSpanLimit && c_span < kSpanLimit;
    // an edge tile can be moved back inside the matrix unless the matrix is shorter than a tile
    // (packed B: columns come in whole panels, so only rows move)
    const bool can_shift = (!m_edge || q.M >= T::BM) && (!n_edge || (T::BMODE != B_PACKED && q.N >= T::BN));
    if (!m_edge && !n_edge && offsets_fit_32) gemm_tile<T, 0>(q, lds, batch, tm, tn);
    else if (can_shift && (m_edge || n_edge) && offsets_fit_32) gemm_tile<T, 3>(q, lds, batch, tm, tn);
    else if (T::BMODE == B_NN && n_edge) {
        if constexpr (T::BMODE == B_NN && T::BN <= 32) {
            if (q.N % 4 == 0) {
                gemm_tile<T, 5>(q, lds, batch, tm, tn);
                return;
            }
        }
        gemm_tile<T, 2>(q, lds, batch, tm, tn);
    }
    else if (T::AMODE != A_MK || offsets_fit_32) gemm_tile<T, 1>(q, lds, batch, tm, tn);
    else if constexpr (T::AMODE == A_MK) gemm_tile<T, 4>(q, lds, batch, tm, tn);
}

// The tile shape that computes one 32 x 32 block of a tail tile of shape T (see KArgs::quad); void
// for shapes whose tails are split along K only.
template <class T, bool = (T::BM * T::BN <= 128 * 64 && T::THREADS == 256 && T::WGK == 1)> struct QuadOf { typedef void type; };
template <class T> struct QuadOf<T, true> { typedef Tile<32, 32, 64, 1, 1, T::BMODE, T::OCC, 2, T::AMODE, 4> type; };

// The strip of a product (see KArgs): C[i][n0 + s] = sum_k A[i][k] * opB[k][n0 + s] for s < S <= kStripMax, A
// stored M x K.  A wave takes R consecutive rows of C, a workgroup of four waves 4R; its lanes stride over k 16
// bytes of A at a time, each lane multiplies its four k against the columns of B, and at the end the 64
// partial sums of every (row, column) are added across the lanes in a fixed order, so the result does not
// depend on the launch.  K is walked in chunks of 256 * BATCH.
// The workgroup shares its compute unit with a tile whose waves issue one matrix instruction after the
// other; measured, a wave beside them gets to issue about one instruction of any kind per matrix instruction
// (64 cycles), whatever its priority: what the strip costs is the number of instructions a wave executes.
// So the code is straight-line: four (S <= 4) or eight columns are carried whatever S is, in groups of four
// that end at column N (columns n0 + S - 4 .. N - 1, and for S > 4 also n0 .. n0 + 3; a column carried twice or
// one that belongs to the tiles is computed and not stored), so that every 16 bytes read from a row of B lie
// inside that row, and the ragged ends along k are left to the range check of buffer descriptors (a dword at or
// beyond the range reads as zero, dword by dword, without a branch or a select).  With B stored N x K a lane
// reads its columns straight from memory (16 bytes along k, as for A); with B stored K x N the workgroup brings
// the columns of a chunk into LDS once for its four waves, two lanes per row of B (one per row for S <= 4).
// The strip is spread over as many workgroups as there are compute units (R = 1 up to 512 rows).  Its waves run
// at the default priority: raised, they went ahead of the tiles' own set-up on the same SIMDs and delayed the tiles'
// first requests (ragged workload 20.1 us against 19.6).
constexpr int kStripMax = 8;
template <int BMODE, int R, bool WIDE>
__device__ __forceinline__ void strip_rows(const KArgs &p, float *lds, const int wg)
{
    for (int i = 0; i < p.strip_wait; ++i) __builtin_amdgcn_s_sleep(16);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int S = p.strip_cols, n0 = p.strip_n0, K = p.K, M = p.M;
    const int r0 = (wg * 4 + wave) * R;
    constexpr int NS = WIDE ? 8 : 4;               // columns carried
    constexpr int FLAGS = 0x00020000;              // 32-bit data
    // carried column s is column c0 + s (s < 4) or c1 + s - 4 of C
    const int c0 = (S >= 4) ? n0 : n0 + S - 4, c1 = n0 + S - 4;
    const unsigned row_bytes = 4u * (unsigned)K;   // (K < 2^30 where a strip is planned)
    __amdgpu_buffer_rsrc_t xr[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const int r = (r0 + j < M) ? (r0 + j) : (M - 1);          // rows past the end repeat the last one; not stored
        xr[j] = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(uniform_pointer(p.A + (int64_t)r * p.lda)), 0, (int)row_bytes, FLAGS);
    }
    float acc[NS][R];
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int j = 0; j < R; ++j) acc[s][j] = 0.f;
    auto load16 = [&](const __amdgpu_buffer_rsrc_t &rsrc, unsigned byte_offset) {
        return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)byte_offset, 0, 0));
    };
    if constexpr (BMODE == B_NT) {
        constexpr int BATCH = 2, KC = 256 * BATCH;
        __amdgpu_buffer_rsrc_t yr[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int col = (s < 4) ? c0 + s : c1 + s - 4;
            yr[s] = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(uniform_pointer(p.B + (int64_t)col * p.ldb)), 0, (int)row_bytes, FLAGS);
        }
        for (int k0 = 0; k0 < K; k0 += KC) {
            const unsigned off = 4u * (unsigned)(k0 + 4 * lane);
            v4f xv[BATCH][R], yv[BATCH][NS];
#pragma unroll
            for (int it = 0; it < BATCH; ++it) {
#pragma unroll
                for (int j = 0; j < R; ++j) xv[it][j] = load16(xr[j], off + 1024u * it);
#pragma unroll
                for (int s = 0; s < NS; ++s) yv[it][s] = load16(yr[s], off + 1024u * it);
            }
            if (k0 == 0) GEMMF32_STAMP(p, 2);
#pragma unroll
            for (int it = 0; it < BATCH; ++it)
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int s = 0; s < NS; ++s)
#pragma unroll
                        for (int j = 0; j < R; ++j) acc[s][j] = __builtin_fmaf(xv[it][j][e], yv[it][s][e], acc[s][j]);
        }
    } else {
        constexpr int BATCH = (R == 4) ? 2 : 4;    // groups of 256 k per chunk (what the registers hold)
        constexpr int KC = 256 * BATCH, QUARTER = KC / 4;
        // LDS word address of (k, s) within a chunk: (((s / 4) * 4 + k % 4) * QUARTER + k / 4) * 4 + s % 4: the 64 lanes
        // of a wave, which hold consecutive groups of four k, read consecutive 16-byte pieces
        constexpr int ROWS = WIDE ? 128 : 256;     // rows of B the workgroup fetches per request
        constexpr int NY = KC / ROWS;
        const int h = WIDE ? (tid & 1) : 0, ky0 = WIDE ? (tid >> 1) : tid;
        // the lane's position in a chunk of B, from the chunk's first row at column c0
        const unsigned y_off = 4u * ((unsigned)ky0 * (unsigned)p.ldb + (unsigned)(h ? c1 - c0 : 0));
        const unsigned y_step = 4u * (unsigned)ROWS * (unsigned)p.ldb;       // (ldb < 2^20 where a strip is planned)
        float *y_dst = lds + (((h << 2) + (ky0 & 3)) * QUARTER + (ky0 >> 2)) * 4;
        const float *y_src = lds + lane * 4;
        for (int k0 = 0; k0 < K; k0 += KC) {
            const unsigned off = 4u * (unsigned)(k0 + 4 * lane);
            v4f xv[BATCH][R];
#pragma unroll
            for (int it = 0; it < BATCH; ++it)
#pragma unroll
                for (int j = 0; j < R; ++j) xv[it][j] = load16(xr[j], off + 1024u * it);
            // B from row k0 on: its range ends behind column N of row K - 1, so rows from K on read as zeros
            const int64_t left = ((int64_t)(K - 1 - k0) * p.ldb + (n0 + S - c0)) * 4;
            const __amdgpu_buffer_rsrc_t br = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<float *>(uniform_pointer(p.B + (int64_t)k0 * p.ldb + c0)), 0,
                (int)(unsigned)(left < 0xFFFFFFFFLL ? left : 0xFFFFFFFFLL), FLAGS);
            v4f yv[NY];
#pragma unroll
            for (int u = 0; u < NY; ++u) yv[u] = load16(br, y_off + y_step * u);
            if (k0 > 0) __syncthreads();           // the chunk before has been read
#pragma unroll
            for (int u = 0; u < NY; ++u) *reinterpret_cast<v4f *>(y_dst + u * (ROWS / 4) * 4) = yv[u];
            __syncthreads();
            if (k0 == 0) GEMMF32_STAMP(p, 2);
#pragma unroll
            for (int it = 0; it < BATCH; ++it)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v4f y[NS / 4];
#pragma unroll
                    for (int g = 0; g < NS / 4; ++g)
                        y[g] = *reinterpret_cast<const v4f *>(y_src + (((g << 2) + e) * QUARTER + 64 * it) * 4);
#pragma unroll
                    for (int s = 0; s < NS; ++s)
#pragma unroll
                        for (int j = 0; j < R; ++j) acc[s][j] = __builtin_fmaf(xv[it][j][e], y[s >> 2][s & 3], acc[s][j]);
                }
        }
    }
    GEMMF32_STAMP(p, 3);
    // Sum over the lanes: value v = R * s + j, NV = NS * R of them.  Each of the first log2(NV) steps halves the
    // number of values a lane carries: the lanes whose bit is clear keep the lower half and receive their
    // partner's partial sums of it, the others the upper half; then a lane carries value
    // lane >> (6 - log2(NV)), and the remaining steps add the lanes that carry the same value.  A fixed
    // order of additions, and NV - 1 + (6 - log2(NV)) exchanges instead of 6 per value.
    constexpr int NV = NS * R;
    float vals[NV];
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int j = 0; j < R; ++j) vals[R * s + j] = acc[s][j];
    int bit = 32;
#pragma unroll
    for (int half = NV / 2; half >= 1; half >>= 1, bit >>= 1) {
        const bool upper = (lane & bit) != 0;
#pragma unroll
        for (int i = 0; i < half; ++i) {
            // both values are read before the choice: with the reads inside the two arms the compiler selects
            // the index instead and walks the whole array for every access
            const float lo = vals[i], hi = vals[i + half];
            const float keep = upper ? hi : lo;
            const float send = upper ? lo : hi;
            vals[i] = keep + __shfl_xor(send, bit, 64);
        }
    }
    float total = vals[0];
    constexpr int SAME = 64 / NV;                  // lanes that carry the same value
#pragma unroll
    for (int off = SAME / 2; off >= 1; off >>= 1) total += __shfl_xor(total, off, 64);
    const int v = lane / SAME, s = v / R, j = v % R;
    const int col = (s < 4) ? c0 + s : c1 + s - 4;
    const bool own = (s < 4) ? (col >= n0) : (col >= n0 + 4);   // not a column of the tiles, and not carried twice
    if (lane % SAME == 0 && own && r0 + j < M) {
        float *dst = p.C + (int64_t)(r0 + j) * p.ldc + col;
        float out = p.alpha * total;
        if (p.beta != 0.f) out += p.beta * *dst;
        *dst = out;
    }
}

template <class T>
__global__ void __launch_bounds__(T::THREADS, T::OCC) gemm_kernel(const KArgs p)
{
    extern __shared__ __align__(16) float lds[];
#ifdef GEMMF32_TIMELINE
    if (p.stamps != nullptr && threadIdx.x == 0 && blockIdx.x < kTimelineMaxWorkgroups) {
        p.stamps[blockIdx.x * 8] = wall_clock64();
        // XCC_ID (hardware register 20) and HW_ID (4): which compute unit the workgroup ran on
        p.stamps[blockIdx.x * 8 + 6] = ((unsigned long long)__builtin_amdgcn_s_getreg(63508) << 32) | (unsigned)__builtin_amdgcn_s_getreg(63492);
    }
#endif
    // All arguments are requested at once: left alone, the compiler fetches each group of them where it is
    // first used, one round trip to the scalar cache after the other along the head of the kernel.
    asm volatile("" ::"s"(p.A), "s"(p.B), "s"(p.C), "s"(p.M), "s"(p.N), "s"(p.K), "s"(p.lda), "s"(p.ldb), "s"(p.ldc));
    asm volatile("" ::"s"(p.sA), "s"(p.sB), "s"(p.sC), "s"(p.tiles_m), "s"(p.tiles_n), "s"(p.group_m), "s"(p.tiles_per_batch),
                 "s"(p.total_tiles), "s"(p.k_total), "s"(p.tail_first), "s"(p.tail_split), "s"(p.quad), "s"(p.strip_first));
    asm volatile("" ::"s"(p.div_batch.magic), "s"(p.div_batch.shift), "s"(p.div_group.magic), "s"(p.div_group.shift),
                 "s"(p.div_rows.magic), "s"(p.div_rows.shift), "s"(p.div_last_rows.magic), "s"(p.div_last_rows.shift),
                 "s"(p.alpha), "s"(p.beta));
    if constexpr (T::THREADS == 256 && T::WGK == 1 && T::AMODE == A_MK && T::BMODE != B_PACKED) {
        if ((int)blockIdx.x >= p.strip_first) {
            const int wg = (int)blockIdx.x - p.strip_first;
            const bool wide = p.strip_cols > 4;
            if (p.strip_r == 1) { if (wide) strip_rows<T::BMODE, 1, true>(p, lds, wg); else strip_rows<T::BMODE, 1, false>(p, lds, wg); }
            else if (p.strip_r == 2) { if (wide) strip_rows<T::BMODE, 2, true>(p, lds, wg); else strip_rows<T::BMODE, 2, false>(p, lds, wg); }
            else { if (wide) strip_rows<T::BMODE, 4, true>(p, lds, wg); else strip_rows<T::BMODE, 4, false>(p, lds, wg); }
            GEMMF32_STAMP(p, 5);
            return;
        }
    }
    int batch, tm, tn;
    KArgs q = p;
    // whole tiles first, then the pieces of the split tail; each kind is spread over the XCDs separately
    const bool is_piece = p.tail_split > 1 && (int)blockIdx.x >= p.tail_first;
    const int logical = is_piece ? 0 : xcd_contiguous_id(blockIdx.x, p.tail_split > 1 ? p.tail_first : p.strip_first);
    if constexpr (!std::is_void<typename QuadOf<T>::type>::value) {
        if (is_piece && p.quad != 0) {
            // one 32 x 32 block of one tile of the last round, by the whole workgroup
            typedef typename QuadOf<T>::type QT;
            constexpr int SUB_N = T::BN / 32;
            const int piece = xcd_contiguous_id(blockIdx.x - p.tail_first, p.strip_first - p.tail_first);
            const int t = piece / p.tail_split, sub = piece - t * p.tail_split;
            tile_coords(p, p.tail_first + t, tm, tn);
            const int qm = tm * (T::BM / 32) + sub / SUB_N, qn = tn * SUB_N + sub % SUB_N;
            if (qm * 32 >= p.M || qn * 32 >= p.N) return;      // a block of an edge tile that lies outside the matrix
            run_tile<QT>(p, lds, 0, qm, qn);
            GEMMF32_STAMP(p, 5);
            return;
        }
    }
    if (is_piece) {
        // one K range of one tile of the last round -> its slot
        const int piece = xcd_contiguous_id(blockIdx.x - p.tail_first, p.strip_first - p.tail_first);
        const int t = piece / p.tail_split, s = piece - t * p.tail_split;
        tile_coords(p, p.tail_first + t, tm, tn);
        batch = 0;
        const int k0 = s * p.tail_k;
        q.K = (p.K - k0 < p.tail_k) ? (p.K - k0) : p.tail_k;
        q.A = p.A + (T::AMODE == A_KM ? (int64_t)k0 * p.lda : (int64_t)k0);
        q.B = p.B + (T::BMODE == B_NN ? (int64_t)k0 * p.ldb : (T::BMODE == B_NT ? (int64_t)k0 : (int64_t)k0 * kPanel));
        // dense BM x BN slot, addressed so that element (m0 + r, n0 + c) lands at r*BN + c
        float *slot = p.tail_slots + (int64_t)piece * (T::BM * T::BN);
        q.C = slot - ((int64_t)tm * T::BM * T::BN + (int64_t)tn * T::BN);
        q.ldc = T::BN;
        q.alpha = 1.f;                 // raw partial sums; the second pass scales
        q.beta = 0.f;
    } else {
        batch = fast_div(logical, p.div_batch);
        tile_coords(p, logical - batch * p.tiles_per_batch, tm, tn);
    }
    run_tile<T>(q, lds, batch, tm, tn);
    GEMMF32_STAMP(p, 5);
}

// Products with at most 8 rows (or columns) whose two operands both have k contiguous (A stored M x K, B
// stored N x K).  Such a product has 2 to 16 flop per byte of its long operand and is bound by reading
// that operand once; the matrix instruction would spend 3/4 or more of its work on padding, and a 32-wide
// tile gives too few workgroups unless K is split.  Here the long operand X (rows x K) is streamed: a wave
// takes kThinRows consecutive rows, its lanes stride over k 16 bytes at a time (a wave reads 1 KB of a row
// per request), multiply with the S rows of the short operand Y (read through the caches) in the vector
// unit, and the 64 partial sums of every (row, s) pair are added by a fixed butterfly over the lanes, so the
// result does not depend on the launch.  Element (r, s) goes to C[r * c_big + s * c_small].
struct ThinArgs {
    const float *X;
    int64_t ldx;
    int rows;
    const float *Y;
    int64_t ldy;
    float *C;
    int64_t c_big, c_small;
    int K;
    float alpha, beta;
};
constexpr int kThinRows = 4;                      // rows of X per wave
constexpr int kThinRowsPerWorkgroup = 4 * kThinRows;

template <int S> __global__ void __launch_bounds__(256) thin_nt_kernel(const ThinArgs p)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r0 = (blockIdx.x * 4 + wave) * kThinRows;
    if (r0 >= p.rows) return;                      // whole waves leave together
    const float *x[kThinRows];
#pragma unroll
    for (int j = 0; j < kThinRows; ++j) {
        const int r = (r0 + j < p.rows) ? (r0 + j) : (p.rows - 1);      // rows past the end repeat the last one; not stored
        x[j] = p.X + (int64_t)r * p.ldx;
    }
    float acc[S][kThinRows];
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int j = 0; j < kThinRows; ++j) acc[s][j] = 0.f;
    const int k4 = p.K & ~3;                       // columns covered 16 bytes at a time
    auto chunk = [&](int k) {                      // k + 3 < k4
        v4f xv[kThinRows], yv[S];
#pragma unroll
        for (int j = 0; j < kThinRows; ++j) xv[j] = load4(x[j] + k);
#pragma unroll
        for (int s = 0; s < S; ++s) yv[s] = load4(p.Y + (int64_t)s * p.ldy + k);
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
            for (int j = 0; j < kThinRows; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[s][j] = __builtin_fmaf(yv[s][e], xv[j][e], acc[s][j]);
    };
    int k = lane * 4;
    for (; k + 256 < k4; k += 512) {               // two requests per row in flight
        chunk(k);
        chunk(k + 256);
    }
    if (k < k4) chunk(k);
    const int kt = k4 + lane;                      // the last K % 4 columns, one per lane
    if (kt < p.K) {
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const float yv = p.Y[(int64_t)s * p.ldy + kt];
#pragma unroll
            for (int j = 0; j < kThinRows; ++j) acc[s][j] = __builtin_fmaf(yv, x[j][kt], acc[s][j]);
        }
    }
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int j = 0; j < kThinRows; ++j) {
            float v = acc[s][j];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
            acc[s][j] = v;
        }
    // lane s * kThinRows + j stores element (r0 + j, s)
    if (lane < S * kThinRows) {
        const int s = lane / kThinRows, j = lane % kThinRows;
        float v = 0.f;
#pragma unroll
        for (int ss = 0; ss < S; ++ss)
#pragma unroll
            for (int jj = 0; jj < kThinRows; ++jj)
                if (ss == s && jj == j) v = acc[ss][jj];
        if (r0 + j < p.rows) {
            float *dst = p.C + (int64_t)(r0 + j) * p.c_big + (int64_t)s * p.c_small;
            float out = p.alpha * v;
            if (p.beta != 0.f) out += p.beta * *dst;
            *dst = out;
        }
    }
}

// Sums the K ranges of the split tail tiles in ascending k and stores them into C.
// One wave per (tail tile, 256-element chunk of the tile), so that even a few tiles spread over the chip.
static __global__ void __launch_bounds__(64) tail_reduce_kernel(const KArgs p, int BM, int BN)
{
    const int chunks_per_tile = BM * BN / 256;
    const int t = blockIdx.x / chunks_per_tile, chunk = blockIdx.x % chunks_per_tile;
    int tm, tn;
    tile_coords(p, p.tail_first + t, tm, tn);
    const int e = chunk * 256 + threadIdx.x * 4;             // element of the tile: row e / BN, 4 columns
    const int r = e / BN, c = e % BN;
    const int gi = tm * BM + r, gj = tn * BN + c;
    if (gi >= p.M || gj >= p.N) return;
    const float *slot = p.tail_slots + (int64_t)t * p.tail_split * (BM * BN) + e;
    float *dst = p.C + (int64_t)gi * p.ldc + gj;
    const float alpha = p.alpha, beta = p.beta;
    if (gj + 3 < p.N) {
        v4f acc = *reinterpret_cast<const v4f *>(slot);
#pragma unroll 8
        for (int s = 1; s < p.tail_split; ++s) acc += *reinterpret_cast<const v4f *>(slot + (int64_t)s * (BM * BN));
        acc *= alpha;
        if (beta != 0.f) acc += beta * *reinterpret_cast<const v4f_g *>(dst);
        *reinterpret_cast<v4f_g *>(dst) = acc;
    } else {
        for (int j = 0; gj + j < p.N; ++j) {
            float acc = slot[j];
            for (int s = 1; s < p.tail_split; ++s) acc += slot[(int64_t)s * (BM * BN) + j];
            acc *= alpha;
            if (beta != 0.f) acc += beta * dst[j];
            dst[j] = acc;
        }
    }
}

// Batched 64x64x64 products (one product = 48 KB of traffic for 0.5 MFLOP: bound by HBM, not by the
// matrix pipe).  A workgroup of 4 waves (one 32x32 block each) walks products w, w + grid, ...;
// the operands of product i+1 are in flight from global memory while product i is multiplied out
// of LDS, and C is stored straight from the accumulators.  Two LDS buffers, one barrier per product.
struct BatchArgs {
    const float *A;
    const float *B;
    float *C;
    int64_t lda, ldb, ldc;
    int64_t sA, sB, sC;
    int batch;
};

template <int BMODE>   // B_NN or B_NT
__global__ void __launch_bounds__(256, 2) batched64_kernel(const BatchArgs p)
{
    constexpr int SA = 68;                                  // A (and N x K stored B) rows: 64 + 4 pad
    constexpr int SB = (BMODE == B_NT) ? 68 : 64;
    constexpr int A_TILE = 64 * SA, B_TILE = 64 * SB, STAGE = A_TILE + B_TILE;
    extern __shared__ __align__(16) float lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int wm0 = (wave >> 1) * 32, wn0 = (wave & 1) * 32;

    // load slots: 4 chunks of A and 4 of B per thread, 16 bytes each
    int64_t ga[4], gb[4];
    int sa[4], sb[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int f = tid + r * 256;
        const int row = f >> 4, c = (f & 15) * 4;           // 16 chunks per 64-float row
        ga[r] = (int64_t)row * p.lda + c;
        sa[r] = row * SA + c;
        gb[r] = (int64_t)row * p.ldb + c;
        sb[r] = row * SB + c;
    }
    v4f ra[4], rb[4];
    auto load_product = [&](int b) {
        const float *A = p.A + (int64_t)b * p.sA;
        const float *B = p.B + (int64_t)b * p.sB;
#pragma unroll
        for (int r = 0; r < 4; ++r) ra[r] = load4(A + ga[r]);
#pragma unroll
        for (int r = 0; r < 4; ++r) rb[r] = load4(B + gb[r]);
    };

    const int a_frag = (wm0 + l32) * SA + 4 * half;
    const int b_frag = (BMODE == B_NT) ? (A_TILE + (wn0 + l32) * SB + 4 * half)
                                       : (A_TILE + 4 * half * SB + wn0 + l32);
    struct Frag { v4f a; float b[4]; };
    auto read_frag = [&](Frag &fr, const float *base, int g) {
        fr.a = *reinterpret_cast<const v4f *>(base + a_frag + 8 * g);
        if constexpr (BMODE == B_NT) {
            const v4f t = *reinterpret_cast<const v4f *>(base + b_frag + 8 * g);
#pragma unroll
            for (int e = 0; e < 4; ++e) fr.b[e] = t[e];
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) fr.b[e] = base[b_frag + (8 * g + e) * SB];
        }
    };

    int b = blockIdx.x;
    if (b >= p.batch) return;
    load_product(b);
    int cur = 0;
    for (; b < p.batch; b += gridDim.x) {
        float *stage = lds + cur * STAGE;
#pragma unroll
        for (int r = 0; r < 4; ++r) *reinterpret_cast<v4f *>(stage + sa[r]) = ra[r];
#pragma unroll
        for (int r = 0; r < 4; ++r) *reinterpret_cast<v4f *>(stage + A_TILE + sb[r]) = rb[r];
        lds_barrier();
        const int nb = b + (int)gridDim.x;
        if (nb < p.batch) load_product(nb);                 // in flight during the multiply

        v16f acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
        Frag f0, f1;
        read_frag(f0, stage, 0);
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            Frag &now = (g & 1) ? f1 : f0;
            Frag &next = (g & 1) ? f0 : f1;
            if (g + 1 < 8) read_frag(next, stage, g + 1);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(now.a[e], now.b[e], acc, 0, 0, 0);
        }
        float *C = p.C + (int64_t)b * p.sC;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int gi = wm0 + 8 * (v / 4) + 4 * half + (v % 4);
            C[(int64_t)gi * p.ldc + wn0 + l32] = acc[v];
        }
        cur ^= 1;
    }
}

// Split-K second pass: C[i][j] = alpha * (sum of the S partial products W[s][i][j], dense M x N
// each) + beta * C[i][j].  SL lanes share one group of 4 adjacent columns: lane p adds the partials
// p, p + SL, p + 2*SL, ... in ascending order, then the SL lane sums are combined by a fixed
// butterfly, so the order of the additions depends on (S, SL) only, never on how the first pass
// was scheduled; with many partials and a small output the loads of one element are in flight
// together instead of one after the other.  beta == 0: C is not read.
template <int SL>
static __global__ void __launch_bounds__(256) splitk_reduce_kernel(const float *__restrict__ W, float *__restrict__ C,
                                                                    int M, int N, int64_t ldc, int S, float alpha,
                                                                    float beta)
{
    const int64_t mn = (int64_t)M * N;
    const int n4 = (N + 3) / 4;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t chunk = gid / SL;
    const int part = (int)(gid % SL);
    if (chunk >= (int64_t)M * n4) return;              // whole groups of SL lanes leave together
    const int i = (int)(chunk / n4), j = (int)(chunk % n4) * 4;
    const float *src = W + (int64_t)i * N + j;
    float *dst = C + (int64_t)i * ldc + j;
    const bool whole = (j + 3 < N);
    v4f acc = {0.f, 0.f, 0.f, 0.f};
    if (whole) {
#pragma unroll 4
        for (int s = part; s < S; s += SL) acc += load4(src + s * mn);
    } else {
        for (int s = part; s < S; s += SL)
            for (int c = 0; j + c < N; ++c) acc[c] += src[s * mn + c];
    }
#pragma unroll
    for (int off = SL / 2; off >= 1; off /= 2) {
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] += __shfl_xor(acc[c], off, 64);
    }
    if (part != 0) return;
    acc *= alpha;
    if (whole) {
        if (beta != 0.f) acc += beta * load4(dst);
        *reinterpret_cast<v4f_g *>(dst) = acc;
    } else {
        for (int c = 0; j + c < N; ++c) dst[c] = (beta != 0.f) ? acc[c] + beta * dst[c] : acc[c];
    }
}

// Array packing (Section 6.1): Bp[x][y][z] = opB[y][x*kPanel + z], zero beyond column N.
// B stored K x N: a re-laid-out copy.  One thread moves four 16-byte pieces (all four loads are
// issued before the first store); a piece never straddles a panel because kPanel % 4 == 0.
static __global__ void __launch_bounds__(256) pack_b_kernel(const float *__restrict__ B, float *__restrict__ Bp,
                                                      int N, int K, int64_t ldb, int64_t total_f4)
{
    constexpr int F4_ROW = kPanel / 4;
    v4f v[4];
    int64_t f[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[i] = (int64_t)blockIdx.x * 1024 + i * 256 + threadIdx.x;
        v[i] = v4f{0.f, 0.f, 0.f, 0.f};
        if (f[i] < total_f4) {
            const int z = (int)(f[i] % F4_ROW) * 4;
            const int64_t xy = f[i] / F4_ROW;
            const int y = (int)(xy % K);
            const int col = (int)(xy / K) * kPanel + z;
            const float *src = B + (int64_t)y * ldb + col;
            if (col + 3 < N) {
                v[i] = load4(src);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (col + e < N) v[i][e] = src[e];
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (f[i] < total_f4) *reinterpret_cast<v4f *>(Bp + f[i] * 4) = v[i];
}

// B stored N x K: the packing is a transpose.  A workgroup moves a 64 (columns of B) x 64 (k)
// block through LDS: 16-byte global reads along k, 16-byte global writes along z, 4-byte LDS
// accesses on an odd row stride (at most 2-way bank conflicts either way).
static __global__ void __launch_bounds__(256) pack_b_transposed_kernel(const float *__restrict__ B, float *__restrict__ Bp,
                                                                 int N, int K, int64_t ldb, int k_blocks)
{
    constexpr int S = 65;
    __shared__ float t[64 * S];                    // t[k][n]
    const int kb = blockIdx.x % k_blocks;
    const int nb = blockIdx.x / k_blocks;          // 64-column block: panel nb / 2, half nb % 2
    const int n0 = nb * 64, k0 = kb * 64;
    const int tid = threadIdx.x;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int f = tid + r * 256;
        const int n = f >> 4, k = (f & 15) * 4;    // 16 pieces per row of 64 k
        const int gn = n0 + n, gk = k0 + k;
        v4f v = {0.f, 0.f, 0.f, 0.f};
        if (gn < N) {
            const float *src = B + (int64_t)gn * ldb + gk;
            if (gk + 3 < K) {
                v = load4(src);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (gk + e < K) v[e] = src[e];
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) t[(k + e) * S + n] = v[e];
    }
    __syncthreads();
    float *dst_panel = Bp + (int64_t)(nb >> 1) * K * kPanel + (nb & 1) * 64;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int f = tid + r * 256;
        const int k = f >> 4, n = (f & 15) * 4;    // 16 pieces per row of 64 columns
        if (k0 + k < K) {
            v4f v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = t[k * S + n + e];
            *reinterpret_cast<v4f *>(dst_panel + (int64_t)(k0 + k) * kPanel + n) = v;
        }
    }
}

}  // namespace gemmf32
