// Optimisation ladder: the same product C = A*B (Section 6.1) built as a sequence of kernels, each
// adding one class of optimisation, mirroring the seven versions whose run times the paper plots
// for its CPU (Section 6.1 schedules, Section 6.6 figure): baseline, blocking, vectorization, loop
// permutation, array packing, cache blocks, parallel.  What each class becomes on this chip:
//
//   0 baseline          one thread per element of C, operands straight from global memory
//   1 blocking          64x64 tile of C per workgroup of four waves, K in slabs of 32 held in LDS, scalar FMAs
//   2 vectorization     the same workgroup; each wave's 32x32 block runs on the matrix unit (fp32 MFMA)
//   3 loop permutation  k-major operand order in LDS: padded rows, a lane reads 16 bytes = 4 MFMA steps
//   4 array packing     B comes from packed panels (packedB[N/P][K][P]); its rows are linear in memory
//   5 cache blocks      accumulators blocked in registers (64x64 per wave, 128x128 per workgroup),
//                       LDS double buffered, next slab in flight while the current one multiplies
//   6 parallel          the production kernels: tile chosen per shape to fill 256 compute units,
//                       XCD-aware tile walk, software-pipelined issue order
//
// Levels 0-5 are deliberately plain; they exist to be measured, not to be fast.  All are correct
// for any M, N, K and any leading dimensions (per-element bounds checks).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gemmf32_ladder {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kPanel = 128;   // same panel width as pack_b

struct Args {
    const float *A;
    const float *B;      // row-major K x N, or the packed panels for levels that use them
    float *C;
    int M, N, K;
    int64_t lda, ldb, ldc;
};

// element (k, j) of B, zero outside the matrix
template <bool PACKED> __device__ __forceinline__ float load_b(const Args &p, int k, int j)
{
    if (k >= p.K || j >= p.N) return 0.f;
    if (PACKED) return p.B[((int64_t)(j / kPanel) * p.K + k) * kPanel + (j % kPanel)];
    return p.B[(int64_t)k * p.ldb + j];
}
__device__ __forceinline__ float load_a(const Args &p, int i, int k)
{
    return (i < p.M && k < p.K) ? p.A[(int64_t)i * p.lda + k] : 0.f;
}

// ---- 0: baseline ------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) level0_baseline(const Args p)
{
    const int j = blockIdx.x * 16 + (threadIdx.x & 15);
    const int i = blockIdx.y * 16 + (threadIdx.x >> 4);
    if (i >= p.M || j >= p.N) return;
    float acc = 0.f;
    for (int k = 0; k < p.K; ++k) acc += p.A[(int64_t)i * p.lda + k] * p.B[(int64_t)k * p.ldb + j];
    p.C[(int64_t)i * p.ldc + j] = acc;
}

// Levels 1 to 4 share one decomposition, so that each differs from the one before in a single respect:
// a 64x64 tile of C per workgroup of 256 threads (four waves), K in slabs of 32 held in LDS, one barrier
// pair per slab, nothing in flight while a slab is multiplied.

// ---- 1: blocking --------------------------------------------------------------------------------
// Each thread a 4x4 patch of the tile; scalar FMAs in the vector unit.
__global__ void __launch_bounds__(256) level1_blocking(const Args p)
{
    __shared__ float As[64][33], Bs[32][65];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    float acc[4][4];
    for (int a = 0; a < 4; ++a)
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.f;
    for (int k0 = 0; k0 < p.K; k0 += 32) {
        for (int e = threadIdx.x; e < 2048; e += 256) {
            As[e >> 5][e & 31] = load_a(p, m0 + (e >> 5), k0 + (e & 31));
            Bs[e >> 6][e & 63] = load_b<false>(p, k0 + (e >> 6), n0 + (e & 63));
        }
        __syncthreads();
        for (int k = 0; k < 32; ++k) {
            float a[4], b[4];
            for (int i = 0; i < 4; ++i) {
                a[i] = As[ty + 16 * i][k];
                b[i] = Bs[k][tx + 16 * i];
            }
            for (int i = 0; i < 4; ++i)
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
        __syncthreads();
    }
    for (int a = 0; a < 4; ++a)
        for (int b = 0; b < 4; ++b) {
            const int i = m0 + ty + 16 * a, j = n0 + tx + 16 * b;
            if (i < p.M && j < p.N) p.C[(int64_t)i * p.ldc + j] = acc[a][b];
        }
}

// D register v of lane (l32, half) of a 32x32x2 fp32 MFMA is D[8*(v/4) + 4*half + v%4][l32]
__device__ __forceinline__ void store_block(const Args &p, const v16f &acc, int i0, int j0, int l32, int half)
{
    for (int v = 0; v < 16; ++v) {
        const int i = i0 + 8 * (v / 4) + 4 * half + (v % 4), j = j0 + l32;
        if (i < p.M && j < p.N) p.C[(int64_t)i * p.ldc + j] = acc[v];
    }
}

// ---- 2: vectorization -----------------------------------------------------------------------------
// The same tile and slabs; each wave's 32x32 block runs on the matrix unit (fp32 MFMA) instead of 1024
// scalar FMAs per k.  Operands lie in LDS in their memory order (A[i][k], B[k][j]); each MFMA step reads
// one float of A and one of B per lane.  A is read down a column of the slab: every lane hits the same bank.
__global__ void __launch_bounds__(256) level2_vectorization(const Args p)
{
    __shared__ float As[64][32], Bs[32][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, half = lane >> 5;
    const int wm0 = (wave >> 1) * 32, wn0 = (wave & 1) * 32;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    v16f acc;
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    for (int k0 = 0; k0 < p.K; k0 += 32) {
        for (int e = threadIdx.x; e < 2048; e += 256) {
            As[e >> 5][e & 31] = load_a(p, m0 + (e >> 5), k0 + (e & 31));
            Bs[e >> 6][e & 63] = load_b<false>(p, k0 + (e >> 6), n0 + (e & 63));
        }
        __syncthreads();
        for (int s = 0; s < 16; ++s)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(As[wm0 + l32][2 * s + half], Bs[2 * s + half][wn0 + l32], acc, 0, 0, 0);
        __syncthreads();
    }
    store_block(p, acc, m0 + wm0, n0 + wn0, l32, half);
}

// ---- 3 and 4: loop permutation, array packing -------------------------------------------------------
// As level 2, but A rows are padded (stride 36) and the k order inside a group of 8 is permuted so
// that a lane's four A operands are 16 contiguous bytes (step e pairs columns e and 4+e).
// PACKED: B is read from the packed panels.
template <bool PACKED>
__global__ void __launch_bounds__(256) level34_permuted(const Args p)
{
    __shared__ __align__(16) float As[64][36];
    __shared__ float Bs[32][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, half = lane >> 5;
    const int wm0 = (wave >> 1) * 32, wn0 = (wave & 1) * 32;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    v16f acc;
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    for (int k0 = 0; k0 < p.K; k0 += 32) {
        for (int e = threadIdx.x; e < 2048; e += 256) {
            As[e >> 5][e & 31] = load_a(p, m0 + (e >> 5), k0 + (e & 31));
            Bs[e >> 6][e & 63] = load_b<PACKED>(p, k0 + (e >> 6), n0 + (e & 63));
        }
        __syncthreads();
        for (int g = 0; g < 4; ++g) {
            const v4f a = *reinterpret_cast<const v4f *>(&As[wm0 + l32][8 * g + 4 * half]);
            for (int e = 0; e < 4; ++e)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], Bs[8 * g + 4 * half + e][wn0 + l32], acc, 0, 0, 0);
        }
        __syncthreads();
    }
    store_block(p, acc, m0 + wm0, n0 + wn0, l32, half);
}

// ---- 5: cache blocks ----------------------------------------------------------------------------
// 128x128 tile, 4 waves, each wave a 64x64 block held in four accumulators; slabs of 16; two LDS
// buffers; the next slab is fetched into registers while the current one is multiplied.  B from the
// packed panels.  Plain block order, no issue-order pinning.
__global__ void __launch_bounds__(256) level5_cache_blocks(const Args p)
{
    constexpr int BK = 16, SA = BK + 4;
    __shared__ __align__(16) float As[2][128][SA];
    __shared__ __align__(16) float Bs[2][BK][128];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int wm0 = (wave >> 1) * 64, wn0 = (wave & 1) * 64;
    const int m0 = blockIdx.y * 128, n0 = blockIdx.x * 128;

    v16f acc[2][2];
    for (int a = 0; a < 2; ++a)
        for (int b = 0; b < 2; ++b)
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // each thread stages 8 floats of A (row tid/2, 8 columns) and 8 of B (row tid/16, 8 columns)
    float ra[8], rb[8];
    const int ar = tid >> 1, ac = (tid & 1) * 8;
    const int br = tid >> 4, bc = (tid & 15) * 8;
    auto fetch = [&](int k0) {
        for (int e = 0; e < 8; ++e) {
            ra[e] = load_a(p, m0 + ar, k0 + ac + e);
            rb[e] = load_b<true>(p, k0 + br, n0 + bc + e);
        }
    };
    auto stash = [&](int buf) {
        for (int e = 0; e < 8; ++e) {
            As[buf][ar][ac + e] = ra[e];
            Bs[buf][br][bc + e] = rb[e];
        }
    };
    const int nk = (p.K + BK - 1) / BK;
    if (nk > 0) {
        fetch(0);
        stash(0);
    }
    __syncthreads();
    for (int t = 0; t < nk; ++t) {
        const int cur = t & 1;
        if (t + 1 < nk) fetch((t + 1) * BK);
        for (int g = 0; g < 2; ++g) {
            v4f a[2];
            for (int i = 0; i < 2; ++i) a[i] = *reinterpret_cast<const v4f *>(&As[cur][wm0 + 32 * i + l32][8 * g + 4 * half]);
            for (int e = 0; e < 4; ++e) {
                const float b0 = Bs[cur][8 * g + 4 * half + e][wn0 + l32];
                const float b1 = Bs[cur][8 * g + 4 * half + e][wn0 + 32 + l32];
                for (int i = 0; i < 2; ++i) {
                    acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][e], b0, acc[i][0], 0, 0, 0);
                    acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][e], b1, acc[i][1], 0, 0, 0);
                }
            }
        }
        if (t + 1 < nk) stash(cur ^ 1);
        __syncthreads();
    }
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j) store_block(p, acc[i][j], m0 + wm0 + 32 * i, n0 + wn0 + 32 * j, l32, half);
}

}  // namespace gemmf32_ladder
