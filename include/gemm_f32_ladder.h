/*
 * Optimisation ladder for the fp32 matrix product C = A * B (row-major, no transpose).
 *
 * The paper evaluates its strategies by running seven differently optimised versions of
 * one matrix product and plotting their run times (Section 6.1 lists the versions:
 * baseline, blocking, vectorization, loop permutation, array packing, write cache for
 * blocks, parallel; Section 6.6 shows the figure).  This entry point runs the MI355X
 * counterpart of each version, so that the same ladder can be measured on this chip.
 * Level 6 is the production path (gemm_f32_packed); levels 0-5 are plain kernels that
 * each add one class of optimisation and exist to be measured.
 *
 * Same conventions as gemm_f32.h: device pointers owned by the caller, element strides,
 * C overwritten, nothing outside [0,M) x [0,N) written, asynchronous on the stream the calling thread gave
 * to gemm_f32_ladder_set_stream (default: null stream), 0 on success or a negative
 * gemmf32_status (GEMMF32_EINVAL for an unknown level or bad dimensions, GEMMF32_ENULL for
 * a missing pointer), nothing launched on error.
 *
 *   level 0-3   read B (K x N, ldb >= N); Bp is ignored and may be NULL.
 *   level 4-6   read the packed operand Bp written by pack_b(N, K, B, ...) (Section 6.1,
 *               packedB); B and ldb are ignored.  As in the paper, packing is a separate
 *               loop nest: time pack_b together with these levels to compare like with like.
 */
#ifndef GEMM_F32_LADDER_H
#define GEMM_F32_LADDER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Number of levels (7: levels 0..6). */
int gemm_f32_ladder_levels(void);

/* Static name of a level ("baseline", "blocking", ...; "invalid" outside the range). */
const char *gemm_f32_ladder_name(int level);

int gemm_f32_ladder(int level, int64_t M, int64_t N, int64_t K,
                    const float *A, int64_t lda,
                    const float *B, int64_t ldb,
                    const float *Bp,
                    float *C, int64_t ldc);

/* Stream for later ladder launches (hipStream_t as void*; NULL = null stream). */
int gemm_f32_ladder_set_stream(void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* GEMM_F32_LADDER_H */
