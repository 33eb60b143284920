// What the strategy layer needs from the product's dispatch (gemm_f32.hip).
#pragma once

#include <stdint.h>

namespace gemmf32_host {

struct TileChoice { int bm, bn, bk, waves_m, waves_n, waves_k, split; };   // waves_m x waves_n x waves_k waves per workgroup

// tile shape and K split the cost model picks for one product
TileChoice choose(int64_t M, int64_t N, int64_t K);
// true if a kernel with this tile shape and wave grid was built
bool has_kernel(int bm, int bn, int bk, int waves_m, int waves_n, int waves_k);
// C = A * op(B) with the given tile shape and K split (1: none) instead of the cost model's
int run_forced(int bm, int bn, int bk, int split, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
               const float *B, int64_t ldb, float *C, int64_t ldc, int transB);

}  // namespace gemmf32_host
