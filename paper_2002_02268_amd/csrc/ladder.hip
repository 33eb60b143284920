// C-ABI entry points of the optimisation ladder (see include/gemm_f32_ladder.h).
#include "../../include/gemm_f32.h"
#include "../../include/gemm_f32_ladder.h"

#include "ladder_kernels.hpp"

using namespace gemmf32_ladder;

namespace gemmf32_host {
hipStream_t current_stream();   // the product library's stream of the calling thread (gemm_f32.hip)
}

namespace {

thread_local hipStream_t g_ladder_stream = nullptr;   // per host thread, like the product's

const char *const kNames[7] = {"baseline",      "blocking",     "vectorization", "loop permutation",
                               "array packing", "cache blocks", "parallel"};

unsigned cdiv(int64_t a, int64_t b) { return (unsigned)((a + b - 1) / b); }

}  // namespace

extern "C" {

int gemm_f32_ladder_levels(void) { return 7; }

const char *gemm_f32_ladder_name(int level) { return (level >= 0 && level < 7) ? kNames[level] : "invalid"; }

int gemm_f32_ladder_set_stream(void *hip_stream)
{
    g_ladder_stream = reinterpret_cast<hipStream_t>(hip_stream);
    return GEMMF32_OK;
}

int gemm_f32_ladder(int level, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                    int64_t ldb, const float *Bp, float *C, int64_t ldc)
{
    if (level < 0 || level >= 7) return GEMMF32_EINVAL;
    if (M < 0 || N < 0 || K < 0 || M > 2147483647LL || N > 2147483647LL || K > 2147483647LL) return GEMMF32_EINVAL;
    if (lda < (K > 1 ? K : 1) || ldc < (N > 1 ? N : 1)) return GEMMF32_EINVAL;
    const bool packed = level >= 4;
    if (!packed && ldb < (N > 1 ? N : 1)) return GEMMF32_EINVAL;
    if (M == 0 || N == 0) return GEMMF32_OK;
    if (C == nullptr) return GEMMF32_ENULL;
    if (K > 0 && (A == nullptr || (packed ? Bp : B) == nullptr)) return GEMMF32_ENULL;
    if (C == A || C == B || C == Bp) return GEMMF32_EALIAS;
    if (level == 6) {
        // the product itself, on the ladder's stream; the product's own stream setting is put back
        hipStream_t saved = gemmf32_host::current_stream();
        gemm_f32_set_stream(g_ladder_stream);
        const int rc = gemm_f32_packed(M, N, K, A, lda, Bp, C, ldc);
        gemm_f32_set_stream(saved);
        return rc;
    }
    Args a;
    a.A = A; a.B = packed ? Bp : B; a.C = C;
    a.M = (int)M; a.N = (int)N; a.K = (int)K;
    a.lda = lda; a.ldb = ldb; a.ldc = ldc;
    const int tile = (level == 0) ? 16 : (level == 5 ? 128 : 64);
    const dim3 grid(cdiv(N, tile), cdiv(M, tile));
    if (grid.y > 65535u * 16u) return GEMMF32_EINVAL;
    switch (level) {
    case 0: hipLaunchKernelGGL(level0_baseline, grid, dim3(256), 0, g_ladder_stream, a); break;
    case 1: hipLaunchKernelGGL(level1_blocking, grid, dim3(256), 0, g_ladder_stream, a); break;
    case 2: hipLaunchKernelGGL(level2_vectorization, grid, dim3(256), 0, g_ladder_stream, a); break;
    case 3: hipLaunchKernelGGL(level34_permuted<false>, grid, dim3(256), 0, g_ladder_stream, a); break;
    case 4: hipLaunchKernelGGL(level34_permuted<true>, grid, dim3(256), 0, g_ladder_stream, a); break;
    default: hipLaunchKernelGGL(level5_cache_blocks, grid, dim3(256), 0, g_ladder_stream, a); break;
    }
    return hipGetLastError() == hipSuccess ? GEMMF32_OK : GEMMF32_ELAUNCH;
}

}  // extern "C"
