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
//   * slab t+1 is fetched from global memory into registers while slab t is multiplied,
//     then written to the other LDS buffer: one barrier per slab.
//
// Lane maps of v_mfma_f32_32x32x2_f32 used below (lane l, l32 = l % 32, h = l / 32):
//   A operand: A[i = l32][k = h]      B operand: B[k = h][j = l32]
//   D register v: D[i = 8*(v/4) + 4*h + v%4][j = l32]
// The two k values of one MFMA step may be any two slab columns as long as A and B agree;
// step e of an 8-column group uses columns e (h = 0) and 4 + e (h = 1).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gemmf32 {

typedef float v2f __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

enum BMode : int { B_NN = 0, B_NT = 1, B_PACKED = 2 };

constexpr int kPanel = 128;  // panel width P of the packed-B layout, in elements

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
    int total_tiles;         // tiles_per_batch * batch == gridDim.x
    int n_padded;            // packed B: number of columns present in the buffer
};

template <int N> struct VecOf;
template <> struct VecOf<1> { typedef float type; };
template <> struct VecOf<2> { typedef v2f type; };
template <> struct VecOf<4> { typedef v4f type; };

template <int N> __device__ __forceinline__ float vget(const typename VecOf<N>::type &v, int i) { return v[i]; }
template <> __device__ __forceinline__ float vget<1>(const float &v, int) { return v; }

template <int BM_, int BN_, int BK_, int WGM_, int WGN_, int BMODE_, bool VEC_, int STAGES_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_;
    static constexpr int BMODE = BMODE_, STAGES = STAGES_;
    static constexpr bool VEC = VEC_;
    static constexpr int THREADS = 64 * WGM * WGN;
    static constexpr int WM = BM / WGM, WN = BN / WGN;
    static constexpr int MB = WM / 32, NB = WN / 32;
    static constexpr int SA = BK + 4;                          // A rows in LDS: [BM][SA]
    static constexpr int SB = (BMODE == B_NT) ? (BK + 4) : BN; // B in LDS: [BN][SB] (NT) or [BK][BN]
    static constexpr int A_TILE = BM * SA;
    static constexpr int B_TILE = (BMODE == B_NT) ? BN * SB : BK * BN;
    static constexpr int STAGE_FLOATS = A_TILE + B_TILE;
    static constexpr int LDS_BYTES = STAGES * STAGE_FLOATS * 4;
    static constexpr int A_F4 = BM * BK / 4, A_ITERS = A_F4 / THREADS;
    static constexpr int B_F4 = BN * BK / 4, B_ITERS = B_F4 / THREADS;
    static_assert(BM % (32 * WGM) == 0 && BN % (32 * WGN) == 0, "wave tiles are multiples of 32");
    static_assert(BK % 8 == 0, "a slab holds whole 8-column groups");
    static_assert(A_F4 % THREADS == 0 && B_F4 % THREADS == 0, "loads divide evenly over threads");
    static_assert(NB == 1 || NB == 2 || NB == 4, "NB columns are read as one LDS vector");
    static_assert(BMODE != B_PACKED || BN % kPanel == 0 || kPanel % BN == 0, "tile vs panel");
    static_assert(STAGES == 1 || STAGES == 2, "single or double buffered");
};

// Maps the hardware workgroup id to a tile.  Workgroups are handed to the 8 XCDs round
// robin; ids are renumbered so that each XCD (own L2) receives one contiguous run of the
// tile walk, and the walk goes down `group_m` tile rows before moving one tile column so
// that a run forms a compact rectangle sharing rows of A and columns of B.
__device__ __forceinline__ void decode_tile(const KArgs &p, int &batch, int &tm, int &tn)
{
    const int wg = blockIdx.x;
    const int chunk = p.total_tiles >> 3, rem = p.total_tiles & 7;
    const int x = wg & 7, q = wg >> 3;
    const int logical = x * chunk + (x < rem ? x : rem) + q;
    batch = logical / p.tiles_per_batch;
    const int t = logical - batch * p.tiles_per_batch;
    const int gsz = p.group_m * p.tiles_n;
    const int grp = t / gsz;
    const int first_m = grp * p.group_m;
    const int gm = (p.tiles_m - first_m < p.group_m) ? (p.tiles_m - first_m) : p.group_m;
    const int r = t - grp * gsz;
    tm = first_m + r % gm;
    tn = r / gm;
}

template <class T>
__global__ void __launch_bounds__(T::THREADS) gemm_kernel(const KArgs p)
{
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK;
    constexpr int MB = T::MB, NB = T::NB, SA = T::SA, SB = T::SB;
    constexpr int NTHR = T::THREADS;
    constexpr int A_ITERS = T::A_ITERS, B_ITERS = T::B_ITERS;
    constexpr int A_F4_ROW = BK / 4;                                  // 16-byte chunks per A row
    constexpr int B_F4_ROW = (T::BMODE == B_NT) ? BK / 4 : BN / 4;    // per B row in the slab
    typedef typename VecOf<NB>::type vnb;

    extern __shared__ __align__(16) float lds[];

    int batch, tm, tn;
    decode_tile(p, batch, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const float *__restrict__ A = p.A + (int64_t)batch * p.sA;
    const float *__restrict__ B = p.B + (int64_t)batch * p.sB;
    float *__restrict__ C = p.C + (int64_t)batch * p.sC;
    const int M = p.M, N = p.N, K = p.K;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int wm0 = (wave / T::WGN) * T::WM, wn0 = (wave % T::WGN) * T::WN;

    const bool interior = (m0 + BM <= M) && (n0 + BN <= N);

    v4f ra[A_ITERS], rb[B_ITERS];

    // ---- global -> registers for the slab starting at column k0 -------------------------
    auto load_a = [&](int k0, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
#pragma unroll
        for (int r = 0; r < A_ITERS; ++r) {
            const int f = tid + r * NTHR;
            const int row = f / A_F4_ROW, c = (f % A_F4_ROW) * 4;
            const int gi = m0 + row, gk = k0 + c;
            const float *src = A + (int64_t)gi * p.lda + gk;
            if (!MASKED && T::VEC) {
                ra[r] = *reinterpret_cast<const v4f *>(src);
            } else if (!MASKED) {
                ra[r] = v4f{src[0], src[1], src[2], src[3]};
            } else {
                v4f v = {0.f, 0.f, 0.f, 0.f};
                if (gi < M) {
                    if (T::VEC && gk + 3 < K) {
                        v = *reinterpret_cast<const v4f *>(src);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (gk + e < K) v[e] = src[e];
                    }
                }
                ra[r] = v;
            }
        }
    };
    auto load_b = [&](int k0, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
#pragma unroll
        for (int r = 0; r < B_ITERS; ++r) {
            const int f = tid + r * NTHR;
            const int row = f / B_F4_ROW, c = (f % B_F4_ROW) * 4;
            if (T::BMODE == B_NT) {
                // B stored N x K: row = column of C, c = offset along k
                const int gj = n0 + row, gk = k0 + c;
                const float *src = B + (int64_t)gj * p.ldb + gk;
                if (!MASKED && T::VEC) {
                    rb[r] = *reinterpret_cast<const v4f *>(src);
                } else if (!MASKED) {
                    rb[r] = v4f{src[0], src[1], src[2], src[3]};
                } else {
                    v4f v = {0.f, 0.f, 0.f, 0.f};
                    if (gj < N) {
                        if (T::VEC && gk + 3 < K) {
                            v = *reinterpret_cast<const v4f *>(src);
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (gk + e < K) v[e] = src[e];
                        }
                    }
                    rb[r] = v;
                }
            } else if (T::BMODE == B_NN) {
                // B stored K x N: row = offset along k, c = column offset
                const int gk = k0 + row, gj = n0 + c;
                const float *src = B + (int64_t)gk * p.ldb + gj;
                if (!MASKED && T::VEC) {
                    rb[r] = *reinterpret_cast<const v4f *>(src);
                } else if (!MASKED) {
                    rb[r] = v4f{src[0], src[1], src[2], src[3]};
                } else {
                    v4f v = {0.f, 0.f, 0.f, 0.f};
                    if (gk < K) {
                        if (T::VEC && gj + 3 < N) {
                            v = *reinterpret_cast<const v4f *>(src);
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (gj + e < N) v[e] = src[e];
                        }
                    }
                    rb[r] = v;
                }
            } else {
                // packed B: [panel][k][kPanel]; columns past N are stored zeros, columns past
                // the last panel do not exist
                const int gk = k0 + row, gj = n0 + c;
                const int panel = gj / kPanel, z = gj % kPanel;
                const float *src = B + ((int64_t)panel * K + gk) * kPanel + z;
                if (!MASKED) {
                    rb[r] = *reinterpret_cast<const v4f *>(src);
                } else {
                    v4f v = {0.f, 0.f, 0.f, 0.f};
                    if (gk < K && gj < p.n_padded) v = *reinterpret_cast<const v4f *>(src);
                    rb[r] = v;
                }
            }
        }
    };
    auto load_slab = [&](int k0) {
        if (interior && k0 + BK <= K) {
            load_a(k0, std::false_type{});
            load_b(k0, std::false_type{});
        } else {
            load_a(k0, std::true_type{});
            load_b(k0, std::true_type{});
        }
    };

    // ---- registers -> LDS -----------------------------------------------------------------
    auto store_slab = [&](int stage) {
        float *As = lds + stage * T::STAGE_FLOATS;
        float *Bs = As + T::A_TILE;
#pragma unroll
        for (int r = 0; r < A_ITERS; ++r) {
            const int f = tid + r * NTHR;
            const int row = f / A_F4_ROW, c = (f % A_F4_ROW) * 4;
            *reinterpret_cast<v4f *>(&As[row * SA + c]) = ra[r];
        }
#pragma unroll
        for (int r = 0; r < B_ITERS; ++r) {
            const int f = tid + r * NTHR;
            const int row = f / B_F4_ROW, c = (f % B_F4_ROW) * 4;
            *reinterpret_cast<v4f *>(&Bs[row * SB + c]) = rb[r];
        }
    };

    // ---- LDS -> MFMA ----------------------------------------------------------------------
    v16f acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    auto compute_slab = [&](int stage) {
        const float *As = lds + stage * T::STAGE_FLOATS;
        const float *Bs = As + T::A_TILE;
        const float *a_base = As + (wm0 + l32) * SA + 4 * half;
#pragma unroll
        for (int g = 0; g < BK / 8; ++g) {
            v4f a[MB];
#pragma unroll
            for (int i = 0; i < MB; ++i)
                a[i] = *reinterpret_cast<const v4f *>(a_base + 32 * i * SA + 8 * g);
            if (T::BMODE == B_NT) {
                // column of block j: wn0 + 32*j + l32
                v4f b[NB];
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    b[j] = *reinterpret_cast<const v4f *>(Bs + (wn0 + 32 * j + l32) * SB + 4 * half + 8 * g);
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int i = 0; i < MB; ++i)
#pragma unroll
                        for (int j = 0; j < NB; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][e], b[j][e], acc[i][j], 0, 0, 0);
            } else {
                // column of block j: wn0 + NB*l32 + j
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const vnb b = *reinterpret_cast<const vnb *>(Bs + (8 * g + e + 4 * half) * SB + wn0 + NB * l32);
#pragma unroll
                    for (int i = 0; i < MB; ++i)
#pragma unroll
                        for (int j = 0; j < NB; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][e], vget<NB>(b, j), acc[i][j], 0, 0, 0);
                }
            }
        }
    };

    // ---- main loop ------------------------------------------------------------------------
    const int nk = (K + BK - 1) / BK;
    if (T::STAGES == 2) {
        if (nk > 0) {
            load_slab(0);
            store_slab(0);
        }
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            const int cur = kt & 1;
            const bool more = kt + 1 < nk;
            if (more) load_slab((kt + 1) * BK);
            compute_slab(cur);
            if (more) store_slab(cur ^ 1);
            __syncthreads();
        }
    } else {
        for (int kt = 0; kt < nk; ++kt) {
            load_slab(kt * BK);
            if (kt > 0) __syncthreads();
            store_slab(0);
            __syncthreads();
            compute_slab(0);
        }
    }

    // ---- epilogue: accumulators -> C (overwrite; masked at the M / N edges) ---------------
#pragma unroll
    for (int i = 0; i < MB; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int gi = m0 + wm0 + 32 * i + 8 * (v / 4) + 4 * half + (v % 4);
            if (T::BMODE == B_NT) {
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const int gj = n0 + wn0 + 32 * j + l32;
                    if (interior || (gi < M && gj < N)) C[(int64_t)gi * p.ldc + gj] = acc[i][j][v];
                }
            } else {
                const int gj = n0 + wn0 + NB * l32;
                float *dst = C + (int64_t)gi * p.ldc + gj;
                bool done = false;
                if constexpr (T::VEC && NB > 1) {
                    if (interior || (gi < M && gj + NB <= N)) {
                        vnb o;
#pragma unroll
                        for (int j = 0; j < NB; ++j) o[j] = acc[i][j][v];
                        *reinterpret_cast<vnb *>(dst) = o;
                        done = true;
                    }
                }
                if (!done) {
#pragma unroll
                    for (int j = 0; j < NB; ++j)
                        if (interior || (gi < M && gj + j < N)) dst[j] = acc[i][j][v];
                }
            }
        }
    }
}

// Array packing (Section 6.1): Bp[x][y][z] = opB[y][x*kPanel + z], zero beyond column N.
// One thread per 4 consecutive z; reads are row-contiguous for B stored K x N.
__global__ void __launch_bounds__(256) pack_b_kernel(const float *__restrict__ B, float *__restrict__ Bp,
                                                      int N, int K, int64_t ldb, int transB, int64_t total_f4)
{
    const int64_t f = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (f >= total_f4) return;
    constexpr int F4_ROW = kPanel / 4;
    const int z = (int)(f % F4_ROW) * 4;
    const int64_t xy = f / F4_ROW;
    const int y = (int)(xy % K);
    const int x = (int)(xy / K);
    v4f v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int col = x * kPanel + z + e;
        if (col < N) v[e] = transB ? B[(int64_t)col * ldb + y] : B[(int64_t)y * ldb + col];
    }
    *reinterpret_cast<v4f *>(Bp + f * 4) = v;
}

}  // namespace gemmf32
