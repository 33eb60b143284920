/*
 * elevate -- a small strategy language that schedules the matrix product, after the paper's
 * ELEVATE (Section 3: strategies, combinators, traversals, normalisation; Section 4: the rewrite of
 * a doubly transposed matrix in a functional array language; Section 6: scheduling primitives --
 * split, reorder, tile, parallel, vectorize, unroll -- written as strategies).  Host side only:
 * programs and strategies are s-expressions, a strategy rewrites a program, and a scheduled loop
 * nest of the product is lowered to the configuration of one of this library's kernels.
 *
 * Programs (terms):  atom | (head arg ...)
 *   functional array language (Section 4):
 *     (let x e0 e1) (fun x e) (app f a) (build n f) (get a i) (length a), variables, integers
 *   image language (Section 5): the binomial filter
 *     (fun img (map2D (fun nbh (reduce add 0 (map mult (zip (join weights2d) (join nbh)))))
 *                     (slide2D 3 1 (pad2D 1 img))))
 *   loop nests over the product's axes (stand-in for the RISE program of Section 6.3):
 *     (loop AXIS EXTENT KIND body), AXIS in M N K, KIND in seq grid wave unroll slab share
 *     (grid: over workgroups; wave: over the waves of a workgroup; unroll: register blocks of a wave;
 *      slab: the K loop staged through LDS; share: a K loop inside a slab whose iterations the waves
 *      of a workgroup take side by side, adding their sums at the end),
 *     leaves mac (one multiply-accumulate) and mfma32x32x2 (one matrix instruction)
 * Strategies:
 *   id fail (seq s ...) (lChoice s ...) (try s) (repeat s)                       Section 3.4
 *   (all s) (one s) (some s)                                                     Section 3.5
 *   (body s) (function s) (argument s) (bodyN n s)                               Section 3.6
 *   (topDown s) (bottomUp s) (allTopDown s) (allBottomUp s) (tryAll s) (normalize s)   3.7, 3.8
 *   rules, Section 4:   buildGet lenBuild letPartialEval letApp funToLet
 *   rules, Section 5:   (separateDot w2d wh wv) (storeRows image|line)
 *   rules, Section 6:   (split AXIS n) (cover AXIS n) interchange (mark KIND) mfma,
 *                       and built from them (tile bm bn) (reorder p0 p1 ...)
 * `one` picks the leftmost sub-term on which its strategy succeeds, so every rewrite is
 * deterministic.
 *
 * All strings are NUL-terminated host strings; output buffers are written up to their capacity
 * and always NUL-terminated (capacity 0: not written).  No call touches the GPU except
 * gemm_f32_scheduled.
 */
#ifndef ELEVATE_H
#define ELEVATE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Return codes: 0 = the strategy succeeded; ELEVATE_FAILED = it failed (the output names the
 * strategy that was unsuccessful, as Failure(s) does in Section 3.2); negative = error. */
enum {
    ELEVATE_OK = 0,
    ELEVATE_FAILED = 1,
    ELEVATE_EPARSE = -1,      /* malformed program or strategy text (output: message) */
    ELEVATE_ENULL = -2,
    ELEVATE_ELIMIT = -6,      /* more than 100000 rule applications: the strategy does not terminate */
    ELEVATE_ELOWER = -7,      /* the nest is not a schedule a kernel can run (output: reason) */
    ELEVATE_ENOKERNEL = -8    /* valid schedule, but no kernel of this library has that shape */
};

/*
 * Applies `strategy` to `program`.  out: the rewritten program (or the failing strategy / error
 * message).  steps (may be NULL): number of rewrite-rule applications.  trace (may be NULL): one
 * line per application, "rule: before => after".
 */
int elevate_rewrite(const char *strategy, const char *program, char *out, size_t out_cap, int *steps,
                    char *trace, size_t trace_cap);

/* 1 if the two programs of the functional language are equal up to renaming of bound variables,
 * 0 if not, ELEVATE_EPARSE / ELEVATE_ENULL on error. */
int elevate_alpha_equal(const char *a, const char *b);

/* Kernel configuration read off a scheduled nest. */
typedef struct {
    int32_t bm, bn, bk;           /* workgroup tile and K slab */
    int32_t waves_m, waves_n;     /* waves per workgroup */
    int32_t wave_m, wave_n;       /* rows / columns of C per wave */
    int32_t split_k;              /* K ranges computed by separate workgroups (1: none) */
    int64_t tiles_m, tiles_n;     /* grid */
    int64_t k_range;              /* length of one K range, a multiple of bk */
    int32_t waves_k;              /* waves of a workgroup that split every K slab between them (1: none) */
} gemmf32_schedule;

/*
 * Starts from the plain nest of the product, (loop M m seq (loop N n seq (loop K k seq mac))),
 * applies `strategy`, and lowers the result.  nest (may be NULL): the scheduled nest as text (or the
 * failing strategy / the reason it cannot be lowered).  Returns ELEVATE_ENOKERNEL (with *out filled
 * in) if the schedule is valid but none of the built kernels has that shape.
 */
int elevate_schedule_gemm(int64_t M, int64_t N, int64_t K, const char *strategy, gemmf32_schedule *out,
                          char *nest, size_t nest_cap);

/*
 * Starts from the 3x3 binomial filter in its naive form (above), applies `strategy`, and reads off
 * which of the three kernels of binomial_f32.h computes the result: *form = 0 naive; 1 separated
 * (after separateDot, row sums stored as a whole image); 2 scanline (row sums stored per line).
 * program (may be NULL): the rewritten program (or the failing strategy / why it has no kernel).
 */
int elevate_schedule_filter(const char *strategy, int *form, char *program, size_t program_cap);

/* The strategy that expresses what the library's own dispatch does for this shape (tile and K
 * split from its cost model), as text that elevate_schedule_gemm accepts. */
int elevate_default_strategy(int64_t M, int64_t N, int64_t K, char *strategy, size_t cap);

/*
 * The library's own dispatch goes through this layer (Section 3.4, left choice; Section 6.5, one schedule per
 * version): for every new shape of a single product it applies
 *     (lChoice (seq admissible_t cheapest_t schedule_t) ...)        one candidate per tile shape t
 * to the plain nest, where admissible_t (may this tile compete for the nest's extents: the dispatch's measured
 * rules) and cheapest_t (does the cost model rank it first) are guards that leave the nest as it is or fail,
 * and schedule_t is the strategy elevate_default_strategy prints; the kernel configuration lowered from the
 * rewritten nest is what the launch is planned from.  applied: how often that happened since the library was
 * loaded; failed: how often no candidate applied or the nest could not be lowered (the cost model's answer
 * was then used as it stood).  Either pointer may be NULL.
 */
void elevate_dispatch_stats(int64_t *applied, int64_t *failed);

/*
 * C = A * op(B) (as gemm_f32: DEVICE pointers, the library's stream, same argument checks and
 * status codes) run with the kernel shape and K split of `s` instead of the library's own choice.
 * GEMMF32_EINVAL if s names a shape no kernel was built for or a split that does not fit K.
 */
int gemm_f32_scheduled(const gemmf32_schedule *s, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
                       const float *B, int64_t ldb, float *C, int64_t ldc, int transB);

#ifdef __cplusplus
}
#endif
#endif /* ELEVATE_H */
