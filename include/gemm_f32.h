/*
 * gemm_f32 -- dense fp32 matrix product C = A * op(B) on one AMD MI355X (gfx950).
 *
 * The operation is the one the paper's deep-learning case study optimises:
 * Section 6.1 states it as C[x,y] = sum_k A[x,k] * B[k,y] with C of shape
 * (M,N); Section 6.3 states the same thing as the RISE program `mm`
 * (a :: M.K.float, b :: K.N.float, each row of a reduced against each column
 * of b by dot = zip, multiply, reduce(+, 0)).  The reduction starts from 0, so
 * C is overwritten (alpha = 1, beta = 0) and its previous contents, NaN
 * included, never influence the result.
 *
 * Conventions shared by every entry point
 *   - All matrix pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or retains them.  The only device memory the
 *     library owns is a workspace for partial products.  Two kinds of products
 *     use it: those whose output is too small to occupy the chip (few tiles,
 *     long K: their K range is split, the partial products go to the workspace
 *     and a second pass sums them in a fixed order), and those whose tile count
 *     leaves a small remainder after whole rounds of 256 tiles (the remainder's
 *     tiles are split along K the same way).  There is one workspace per stream,
 *     so calls on different streams never share one, and calls on one stream
 *     are ordered by the stream.  It is allocated by the first call that needs
 *     it and replaced by a larger one when a later call needs more (at most
 *     256 MiB per stream; GEMMF32_ENOMEM if the allocation fails); no call frees
 *     memory or waits for the device.  gemm_f32_reserve_workspace sizes it ahead
 *     of time, gemm_f32_shutdown releases everything, and gemm_f32_noalloc is the
 *     entry point for callers that must not allocate at all.
 *   - Row-major storage with element strides (BLAS style):
 *       A   M x K, element (i,k) at A[i*lda + k],              lda >= max(K,1)
 *       B   transB == 0: K x N, element (k,j) at B[k*ldb + j], ldb >= max(N,1)
 *           transB != 0: stored N x K (K x N column-major),
 *                        element (k,j) at B[j*ldb + k],        ldb >= max(K,1)
 *           (Section 6.3 reads b through transpose(b) as a view; transB hands
 *            the library storage that already is that view.)
 *       C   M x N, element (i,j) at C[i*ldc + j],              ldc >= max(N,1)
 *   - Elements of C outside [0,M) x [0,N) (the ldc padding) are never written.
 *   - M == 0 or N == 0: success, nothing launched.  K == 0: C is filled with
 *     +0.0 (the empty sum).
 *   - Work is enqueued on the calling thread's stream (gemm_f32_set_stream;
 *     default: the null stream) and the call returns without waiting for it.
 *   - Return value: GEMMF32_OK (0) or a negative gemmf32_status.  On error
 *     nothing has been launched.  C must not be the same pointer as A or B
 *     (GEMMF32_EALIAS); partially overlapping buffers are undefined behaviour.
 *   - Dimensions are limited to 2^31 - 1 and every operand (rows * ld) to 2^40
 *     elements (GEMMF32_EINVAL beyond that).
 *   - Results are deterministic run to run for a fixed shape, strides and
 *     pointer alignment; no floating-point atomics are used.
 *   - The stream setting is per host thread: every thread that calls the
 *     library sets its own stream, and threads on different streams may call
 *     concurrently.  Two threads that use the same stream are ordered only by
 *     the order in which their launches reach the stream.
 */
#ifndef GEMM_F32_H
#define GEMM_F32_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GEMMF32_OK = 0,
    GEMMF32_EINVAL = -1,  /* negative or oversized dimension, stride too small, bad flag */
    GEMMF32_ENULL = -2,   /* a required pointer is NULL */
    GEMMF32_EALIAS = -3,  /* C is the same buffer as A or B */
    GEMMF32_ELAUNCH = -4, /* the HIP runtime refused; see gemm_f32_last_hip_error */
    GEMMF32_ENOMEM = -5,  /* the workspace could not be allocated */
    GEMMF32_ESCRATCH = -6 /* gemm_f32_noalloc: the product needs more scratch than the fixed array holds */
} gemmf32_status;

/*
 * C = A * op(B)  (Section 6.1 compute expression; Section 6.3 `mm`).
 * A, B, C: device pointers, layouts as above.  transB: 0 or 1.
 */
int gemm_f32(int64_t M, int64_t N, int64_t K,
             const float *A, int64_t lda,
             const float *B, int64_t ldb,
             float *C, int64_t ldc, int transB);

/*
 * batch independent products C_b = A_b * op(B_b), X_b = X + b*strideX
 * (element strides; strideC must be >= the extent of one C so that outputs do
 * not overlap -- not checked).  The paper has no batched form; this applies the
 * Section 6.1 definition to each batch, the analogue of mapping the product
 * over an outermost parallel dimension (mapPar, Section 6.2).
 * batch == 0: success, nothing launched.
 */
int gemm_f32_batched(int64_t batch, int64_t M, int64_t N, int64_t K,
                     const float *A, int64_t lda, int64_t strideA,
                     const float *B, int64_t ldb, int64_t strideB,
                     float *C, int64_t ldc, int64_t strideC, int transB);

/*
 * General form:  C = alpha * op(A) * op(B) + beta * C.
 * The paper's product (Section 6.1 / 6.3) is alpha = 1, beta = 0, transA = 0; Section 6.3 reads b
 * through transpose(b) as a view of the caller's array, and transA applies the same view to a.
 * alpha and beta are the usual library scalings layered on that product:
 *     C[i][j] = alpha * (sum_k opA[i][k] * opB[k][j]) + beta * C_old[i][j],
 * the sum in fp32 on the matrix pipe, the scalings and the addition in fp32.
 *   transA == 0: A stored M x K, lda >= max(K,1).   transA == 1: A stored K x M, lda >= max(M,1).
 *   transB, B, ldb, C, ldc: as gemm_f32.
 *   beta == 0: the old contents of C are never read (they may be NaN).  beta != 0: every element of
 *   C in [0,M) x [0,N) is read once and written once; the ldc padding is never touched.
 *   alpha == 0 does not skip the product: NaN or Inf in A or B still reach C, as alpha * sum says.
 *   K == 0: C = beta * C (zeros for beta == 0).
 * Everything else (device pointers, stream, errors, no launch on error, the split-K workspace) as
 * gemm_f32.  The batched form applies it to batch independent products with element strides.
 */
int gemm_f32_ex(int64_t M, int64_t N, int64_t K, float alpha,
                const float *A, int64_t lda, int transA,
                const float *B, int64_t ldb, int transB,
                float beta, float *C, int64_t ldc);
int gemm_f32_ex_batched(int64_t batch, int64_t M, int64_t N, int64_t K, float alpha,
                        const float *A, int64_t lda, int64_t strideA, int transA,
                        const float *B, int64_t ldb, int64_t strideB, int transB,
                        float beta, float *C, int64_t ldc, int64_t strideC);

/*
 * Array packing of B (Section 6.1, the packedB compute expression):
 *     packedB[x][y][z] = B[y][x*P + z],  shape (ceil(N/P), K, P),
 * with P = pack_b_panel_width() (the paper's 32 was its CPU's choice) and the
 * ragged last panel filled with +0.0.
 *   pack_b_panel_width()  P, in elements.
 *   pack_b_size(N,K)      bytes the caller must provide for Bp
 *                         (ceil(N/P)*K*P*4; 0 if N or K is 0 or negative).
 *   pack_b(...)           reads op(B) (device, layout as above) and writes Bp
 *                         (device, 16-byte aligned, caller-owned).  Bp must not
 *                         overlap B.
 */
int64_t pack_b_panel_width(void);
size_t pack_b_size(int64_t N, int64_t K);
int pack_b(int64_t N, int64_t K, const float *B, int64_t ldb, int transB, float *Bp);

/*
 * C = A * B with B given as packedB from pack_b (Section 6.1, the compute
 * expression rewritten on packedB: C[x,y] = sum_k A[x,k]*packedB[y/P][k][y%P]).
 * Bp: device pointer, 16-byte aligned, produced by pack_b for the same (N,K).
 */
int gemm_f32_packed(int64_t M, int64_t N, int64_t K,
                    const float *A, int64_t lda,
                    const float *Bp,
                    float *C, int64_t ldc);

/* Stream for all later launches of the calling host thread (a hipStream_t
 * passed as void*; NULL = null stream).  The caller keeps ownership of the
 * stream. */
int gemm_f32_set_stream(void *hip_stream);

/*
 * Makes the workspace of the calling thread's stream at least `bytes` large
 * now, so that later calls on that stream which need no more than that
 * allocate nothing.  bytes > 256 MiB: GEMMF32_EINVAL.  A product whose K is
 * split into S ranges needs S*M*N*4 bytes (S is chosen so that this stays
 * within 256 MiB); one whose last round is split needs at most 256 tiles'
 * worth of floats (2 MiB for the 64 x 64 tiles, 64 MiB for 256 x 256).
 * Allocates (hipMalloc) unless the workspace is already that large.
 */
int gemm_f32_reserve_workspace(size_t bytes);

/*
 * gemm_f32 for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and the same result, bit for bit, as gemm_f32; the
 * partial products of a split K or a split last round go to a fixed array of
 * gemm_f32_noalloc_scratch_bytes() (32 MiB) in the library's code object, one
 * copy per device, instead of the allocated workspace.  The call allocates and
 * frees nothing.  A product whose split needs more than the array holds is
 * refused with GEMMF32_ESCRATCH and nothing is launched (gemm_f32 serves it).
 * Every call on a device shares that device's array, whatever its stream:
 * calls that may overlap in time on one device race on it and must be ordered
 * by the caller.  Nothing in the array needs clearing between calls: the
 * second pass reads only what the first pass of the same call has written.
 */
int gemm_f32_noalloc(int64_t M, int64_t N, int64_t K,
                     const float *A, int64_t lda,
                     const float *B, int64_t ldb,
                     float *C, int64_t ldc, int transB);
size_t gemm_f32_noalloc_scratch_bytes(void);

/* Static, never-NULL description of a status code. */
const char *gemm_f32_strerror(int status);

/* hipError_t (as int) of the most recent GEMMF32_ELAUNCH / GEMMF32_ENOMEM on this thread, else 0. */
int gemm_f32_last_hip_error(void);

/* Waits for the device, then releases every workspace.  The library stays usable. */
void gemm_f32_shutdown(void);

/*
 * Which kernel variant the dispatcher would run for a shape, as a string such as
 * "t256x256x16/nn/a16", "t64x64x64/nn/a16/splitk32" (K split into 32 ranges) or
 * "t64x64x64/nn/a4/tail16x8" (the 16 tiles of the last round split into 8 K ranges each) or
 * "t64x64x32/nn/a4/quad16" (the 16 tiles of the last round computed as 32 x 32 blocks) or
 * "t64x64x64/nn/a4/strip6" (the last 6 columns of C computed in the vector unit beside the tiles); for
 * diagnostics and benchmarks.  The pointers are only inspected for alignment and may be NULL for
 * "aligned".  The string lives in a per-thread buffer that the next call on the thread overwrites.
 */
const char *gemm_f32_variant_name(int64_t M, int64_t N, int64_t K,
                                  const float *A, int64_t lda,
                                  const float *B, int64_t ldb,
                                  const float *C, int64_t ldc, int transB);

#ifdef __cplusplus
}
#endif
#endif /* GEMM_F32_H */
