/*
 * gemm_f32_testing -- hooks for tests and measurements of the gemm_f32 library.  Nothing here is
 * meant for production callers; the product entry points are in gemm_f32.h.
 */
#ifndef GEMM_F32_TESTING_H
#define GEMM_F32_TESTING_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Overrides of the dispatch (Section 6.5 of the paper lists one schedule per version of the product; the
 * library picks among its kernels by a cost model, and tests need to reach every kernel on every shape).
 * Process-wide; all fields zero except force_tile = -1 is the production setting.  The environment is
 * never consulted.
 *   force_tile     -1, or 0..12: tile 256x256x16, 128x128x16, 64x64x32, 64x64x64, 256x128x16, 128x256x16,
 *                  128x64x32, 64x128x32, 128x32x32, 32x128x32, and 32x32x64, 64x32x64, 32x64x64 with four waves
 *                  sharing each slab
 *   force_split    0, or S in 1..256: K split into S ranges where that fits
 *   no_tail_split  never split the last round
 *   no_quad        split the last round along K only, never into 32 x 32 blocks
 *   no_kshare      the 32x32x64 tile only for outputs at most 32 wide, not for outputs of a few hundred blocks
 *   no_thin        never the vector-unit kernel for products with at most 4 rows or columns
 *   force_thin     that kernel wherever it can run (at most 8 rows or columns, both operands with k contiguous)
 *   no_strip       never the vector-unit strip for the last few columns of C: they take an edge tile column
 *   force_strip    that strip wherever it can run (by default the cost model weighs it against the edge tile column)
 *   strip_rows     0, or 1, 2, 4: rows of C per wave of a strip workgroup, in place of the library's own figure
 *   strip_wait     0, or 1 + the number of 1024-cycle pauses the strip workgroups take before their first load
 *                  (1: none; at most 65), in place of the library's own figure
 * gemm_f32_set_test_hooks(NULL) restores production.  Returns GEMMF32_EINVAL for values out of range
 * (nothing is changed then).  Changing the hooks while another thread is inside a call is a race in the
 * sense that the call may see the old or the new setting, never a mixture that is invalid.
 * gemm_f32_scheduled (elevate.h) is the interface for choosing tile and split per call.
 */
typedef struct {
    int32_t force_tile;
    int32_t force_split;
    int32_t no_tail_split;
    int32_t no_quad;
    int32_t no_kshare;
    int32_t no_thin;
    int32_t force_thin;
    int32_t no_strip;
    int32_t strip_wait;
    int32_t force_strip;
    int32_t strip_rows;
} gemmf32_test_hooks;

int gemm_f32_set_test_hooks(const gemmf32_test_hooks *hooks);

/*
 * Measurement aid: launches 256 workgroups of 4 waves (one wave per SIMD of every compute unit) that
 * issue mfma_per_wave (a multiple of 16) fp32 32x32x2 matrix instructions each on register operands
 * and touch no memory.  One such instruction occupies the matrix pipe for 64 cycles, so
 *     64 * mfma_per_wave / (run time)
 * is the clock the chip sustains under full matrix load, and 256 CUs * 256 flop/cycle times that
 * clock is the matrix peak actually available (the nominal 157.3 TFLOP/s assumes 2.4 GHz).
 * operands: DEVICE pointer to 512 floats; thread t of every workgroup multiplies operands[2t] by
 * operands[2t+1] throughout (the sustained clock depends on the values: zeros draw less power than
 * random numbers, and the chip is power-limited under matrix load).
 * sink: DEVICE pointer to at least one float (never written in practice).  Asynchronous on the
 * calling thread's stream; the caller times it.
 */
int gemm_f32_mfma_rate_probe(int64_t mfma_per_wave, const float *operands, float *sink);

#ifdef __cplusplus
}
#endif
#endif /* GEMM_F32_TESTING_H */
