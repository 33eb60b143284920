// What the strategy layer needs from the product's dispatch (gemm_f32.hip).
#pragma once

#include <stdint.h>

namespace gemmf32_host {

struct TileChoice { int bm, bn, bk, waves_m, waves_n, waves_k, split; };   // waves_m x waves_n x waves_k waves per workgroup
struct ShapeQuery { int64_t batch, M, N, K; int bmode, amode; };           // bmode: 0 K x N, 1 N x K, 2 packed; amode: 0 M x K, 1 K x M

// the tile shapes kernels were built for
int tile_count();
TileChoice tile_shape(int tile);
// may this tile compete for the shape at all (the dispatch's measured rules)?
bool admissible_tile(int tile, const ShapeQuery &q);
// Implemented by the strategy layer, called by the dispatch once per new shape: rewrites the product's loop
// nest with a left choice over the tiles, each guarded by "may compete" and "is the one the cost model ranks
// first (`cheapest`)", and lowers the rewritten nest.  false: no guarded schedule applied or the nest could
// not be lowered.
bool dispatch_by_strategy(const ShapeQuery &q, const TileChoice &cheapest, TileChoice &lowered);
// how often the dispatch built its plan from a lowered nest, and how often that failed (the cost model's
// answer was used as it stood)
void strategy_dispatch_stats(long long *applied, long long *failed);

// tile shape and K split the cost model picks for one product
TileChoice choose(int64_t M, int64_t N, int64_t K);
// true if a kernel with this tile shape and wave grid was built
bool has_kernel(int bm, int bn, int bk, int waves_m, int waves_n, int waves_k);
// C = A * op(B) with the given tile shape and K split (1: none) instead of the cost model's
int run_forced(int bm, int bn, int bk, int split, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
               const float *B, int64_t ldb, float *C, int64_t ldc, int transB);

}  // namespace gemmf32_host
