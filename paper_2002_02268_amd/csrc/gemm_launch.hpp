// Tile variants of the product kernel and their launch.  The instantiations are spread over
// several translation units (gemm_inst_*.hip), one per operand layout, so that they compile in
// parallel; gemm_f32.hip only declares them.
#pragma once

#include "../../include/gemm_f32.h"
#include "gemm_kernels.hpp"

#include <atomic>

namespace gemmf32_host {

using namespace gemmf32;

hipStream_t current_stream();              // the calling thread's stream (gemm_f32_set_stream)
int record_hip_error(hipError_t e);        // remembers e for gemm_f32_last_hip_error; returns GEMMF32_ELAUNCH

// Raises a kernel's dynamic LDS limit once per device.  `done` (one per kernel) holds a bit per device
// ordinal; two threads that both find their bit clear both set the attribute, which is harmless.
inline int ensure_lds_limit(const void *kernel, int bytes, std::atomic<uint64_t> &done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return record_hip_error(e);
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return GEMMF32_OK;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return record_hip_error(e);
    done.fetch_or(bit, std::memory_order_release);
    return GEMMF32_OK;
}

// ---- variants -------------------------------------------------------------------------------
enum TileId : int { T256 = 0, T128 = 1, T64 = 2, TB64 = 3, T256x128 = 4, T128x256 = 5, T128x64 = 6, T64x128 = 7, T128x32 = 8, T32x128 = 9, TQ32 = 10, TQ64x32 = 11, TQ32x64 = 12, NUM_TILES = 13 };

struct TileShape { int bm, bn, bk, waves_m, waves_n, waves_k; const char *name; };   // waves_k: waves that split a slab along k
const TileShape kShapes[NUM_TILES] = {
    {256, 256, 16, 2, 2, 1, "t256x256x16"}, {128, 128, 16, 2, 2, 1, "t128x128x16"}, {64, 64, 32, 2, 2, 1, "t64x64x32"},
    {64, 64, 64, 2, 2, 1, "t64x64x64"},     {256, 128, 16, 2, 2, 1, "t256x128x16"}, {128, 256, 16, 2, 2, 1, "t128x256x16"},
    {128, 64, 32, 2, 2, 1, "t128x64x32"},   {64, 128, 32, 2, 2, 1, "t64x128x32"},   {128, 32, 32, 4, 1, 1, "t128x32x32"},
    {32, 128, 32, 1, 4, 1, "t32x128x32"},   {32, 32, 64, 1, 1, 4, "t32x32x64k4"},   {64, 32, 64, 1, 1, 4, "t64x32x64k4"},
    {32, 64, 64, 1, 1, 4, "t32x64x64k4"}};

template <int ID, int BMODE, int AMODE> struct Variant;
template <int BMODE, int AMODE> struct Variant<T256, BMODE, AMODE> { typedef Tile<256, 256, 16, 2, 2, BMODE, 1, 1, AMODE> type; };
template <int BMODE, int AMODE> struct Variant<T128, BMODE, AMODE> { typedef Tile<128, 128, 16, 2, 2, BMODE, 2, 2, AMODE> type; };
template <int BMODE, int AMODE> struct Variant<T64, BMODE, AMODE> { typedef Tile<64, 64, 32, 2, 2, BMODE, 2, 2, AMODE> type; };
template <int BMODE, int AMODE> struct Variant<TB64, BMODE, AMODE> { typedef Tile<64, 64, 64, 2, 2, BMODE, 2, 2, AMODE> type; };
template <int BMODE, int AMODE> struct Variant<T256x128, BMODE, AMODE> { typedef Tile<256, 128, 16, 2, 2, BMODE, 2, 1, AMODE> type; };
template <int BMODE, int AMODE> struct Variant<T128x256, BMODE, AMODE> { typedef Tile<128, 256, 16, 2, 2, BMODE, 2, 1, AMODE> type; };
template <int BMODE, int AMODE> struct Variant<T128x64, BMODE, AMODE> { typedef Tile<128, 64, 32, 2, 2, BMODE, 2, 2, AMODE> type; };
template <int BMODE, int AMODE> struct Variant<T64x128, BMODE, AMODE> { typedef Tile<64, 128, 32, 2, 2, BMODE, 2, 2, AMODE> type; };
// one 32 x 32 block per wave, four waves along the long side: for products with at most 32 columns (rows)
template <int BMODE, int AMODE> struct Variant<T128x32, BMODE, AMODE> { typedef Tile<128, 32, 32, 4, 1, BMODE, 3, 2, AMODE> type; };
template <int BMODE, int AMODE> struct Variant<T32x128, BMODE, AMODE> { typedef Tile<32, 128, 32, 1, 4, BMODE, 3, 2, AMODE> type; };

// LDS a launch of shape T may need: its own two slab buffers, or those of the tile shape that computes
// the 32 x 32 blocks of its tail tiles
template <class T, class Q = typename QuadOf<T>::type> struct LdsNeed {
    static constexpr int value = T::LDS_BYTES > Q::LDS_BYTES ? T::LDS_BYTES : Q::LDS_BYTES;
};
template <class T> struct LdsNeed<T, void> { static constexpr int value = T::LDS_BYTES; };

// one 32 x 32 block per workgroup, its four waves splitting every slab along k: for outputs at most 32 wide
// whose other side gives the chip enough blocks, so that K needs no split over workgroups and no second pass
template <int BMODE, int AMODE> struct Variant<TQ32, BMODE, AMODE> { typedef Tile<32, 32, 64, 1, 1, BMODE, 3, 2, AMODE, 4> type; };

// the same with two 32 x 32 blocks per workgroup: a quarter fewer operand bytes per flop, half the workgroups
template <int BMODE, int AMODE> struct Variant<TQ64x32, BMODE, AMODE> { typedef Tile<64, 32, 64, 1, 1, BMODE, 2, 2, AMODE, 4> type; };
template <int BMODE, int AMODE> struct Variant<TQ32x64, BMODE, AMODE> { typedef Tile<32, 64, 64, 1, 1, BMODE, 2, 2, AMODE, 4> type; };

template <class T> int launch(const KArgs &a)
{
    static std::atomic<uint64_t> lds_limit_set{0};  // per instantiation
    auto kern = gemm_kernel<T>;
    const int rc = ensure_lds_limit(reinterpret_cast<const void *>(kern), LdsNeed<T>::value, lds_limit_set);
    if (rc != GEMMF32_OK) return rc;
    // blocks of tail tiles only for shapes that have the block kernel: without it the pieces would be
    // taken for K ranges and stored through a slot pointer that was never set
    if (a.quad != 0 && std::is_void<typename QuadOf<T>::type>::value) return GEMMF32_EINVAL;
    // a product whose K fits one slab never touches a second LDS buffer
    int lds_bytes = (a.K <= T::BK) ? T::LDS_BYTES / 2 : T::LDS_BYTES;
    if (a.quad != 0) lds_bytes = LdsNeed<T>::value;
    // waves that share the slabs add their accumulators through LDS at the end
    constexpr int kSumBytes = (T::WGK > 1) ? T::WGK * T::BM * (T::BN + 1) * 4 : 0;
    if (lds_bytes < kSumBytes) lds_bytes = kSumBytes;
    // the strip workgroups need the kernel that contains them, and 32 KB of LDS for B's columns
    if (a.strip_cols > 0 && !(T::THREADS == 256 && T::WGK == 1 && T::AMODE == A_MK && T::BMODE != B_PACKED)) return GEMMF32_EINVAL;
    if (a.strip_cols > 0 && lds_bytes < 32768) lds_bytes = 32768;
    const KArgs &b = a;
    hipLaunchKernelGGL(kern, dim3((unsigned)b.total_tiles), dim3(T::THREADS), lds_bytes, current_stream(), b);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return record_hip_error(e);
    return GEMMF32_OK;
}

template <int BMODE, int AMODE> int launch_tile(int tile, const KArgs &a)
{
    switch (tile) {
    case T256: return launch<typename Variant<T256, BMODE, AMODE>::type>(a);
    case T128: return launch<typename Variant<T128, BMODE, AMODE>::type>(a);
    case T64: return launch<typename Variant<T64, BMODE, AMODE>::type>(a);
    case T256x128: return launch<typename Variant<T256x128, BMODE, AMODE>::type>(a);
    case T128x256: return launch<typename Variant<T128x256, BMODE, AMODE>::type>(a);
    case T128x64: return launch<typename Variant<T128x64, BMODE, AMODE>::type>(a);
    case T64x128: return launch<typename Variant<T64x128, BMODE, AMODE>::type>(a);
    case T128x32: return launch<typename Variant<T128x32, BMODE, AMODE>::type>(a);
    case T32x128: return launch<typename Variant<T32x128, BMODE, AMODE>::type>(a);
    case TQ32: return launch<typename Variant<TQ32, BMODE, AMODE>::type>(a);
    case TQ64x32: return launch<typename Variant<TQ64x32, BMODE, AMODE>::type>(a);
    case TQ32x64: return launch<typename Variant<TQ32x64, BMODE, AMODE>::type>(a);
    default: return launch<typename Variant<TB64, BMODE, AMODE>::type>(a);
    }
}


}  // namespace gemmf32_host
