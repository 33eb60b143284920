/*
 * CPU oracle for the dense fp32 matrix product C = A * op(B).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the GPU path and must never be called from it.
 *
 * What is computed follows the paper's problem statement in Section 6.1
 * (the TVM compute expression: C is (M,N), C[x,y] = sum over k of
 * A[x,k]*B[k,y]) and Section 6.3 (the RISE program mm: a is M.K.float,
 * b is K.N.float, every row of a is paired with every column of b and
 * reduced by dot = zip, multiply, reduce(+, 0)).  The reduction starts from
 * the identity 0, so C is overwritten and an empty sum (K = 0) is 0.
 *
 * Arithmetic: inputs are IEEE binary32 (the paper's `float`).  Each operand is
 * widened to binary64 (exact), each product is formed in binary64 (exact,
 * 24+24 <= 53 significand bits), and the sum runs over k ascending in
 * binary64.  The result stays in binary64.
 *
 * Every function here is pinned by tests that do not go through this file's
 * own formula: exact integer brute force, identity / all-ones closed forms,
 * indicator probes, the transpose identity, associativity with a vector and a
 * library matrix product.  Nothing in this file is "parity unpinned".
 *
 * Layout convention (BLAS-like, element strides):
 *   A is M x K row-major, element (i,k) at A[i*lda + k], lda >= K.
 *   transB == 0: B is K x N row-major, element (k,j) at B[k*ldb + j], ldb >= N.
 *   transB != 0: B is stored N x K row-major (that is K x N column-major),
 *                element (k,j) at B[j*ldb + k], ldb >= K.  The RISE program
 *                of Section 6.3 reads b through transpose(b) as a view; this
 *                is the same view applied to the caller's storage.
 *   C is M x N row-major, element (i,j) at C[i*ldc + j], ldc >= N.
 * Elements of C outside [0,M) x [0,N) are never written.
 */
#include <stddef.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Returns 0 on success, -1 on an invalid dimension / stride / null pointer. */
static int check_args(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
                      const void *B, int64_t ldb, const void *C, int64_t ldc, int transB)
{
    if (M < 0 || N < 0 || K < 0) return -1;
    if (lda < (K > 1 ? K : 1)) return -1;
    if (ldc < (N > 1 ? N : 1)) return -1;
    if (transB ? ldb < (K > 1 ? K : 1) : ldb < (N > 1 ? N : 1)) return -1;
    if (M > 0 && N > 0 && C == NULL) return -1;
    if (M > 0 && N > 0 && K > 0 && (A == NULL || B == NULL)) return -1;
    return 0;
}

/*
 * Section 6.1 / 6.3: C[i][j] = sum_{k=0}^{K-1} A[i][k] * opB[k][j].
 * The loop nest is the definition written out: rows of A, columns of B, then
 * the dot product.  Threads (if any) split the row loop only; each output
 * element is still produced by one thread with k ascending, so the result
 * does not depend on nthreads.  nthreads <= 0 means "one thread".
 */
int oracle_gemm_f32(int64_t M, int64_t N, int64_t K,
                    const float *A, int64_t lda,
                    const float *B, int64_t ldb,
                    double *C, int64_t ldc,
                    int transB, int nthreads)
{
    if (check_args(M, N, K, A, lda, B, ldb, C, ldc, transB) != 0) return -1;
    if (nthreads <= 0) nthreads = 1;
    (void)nthreads;
    int64_t i;
#ifdef _OPENMP
#pragma omp parallel for num_threads(nthreads) schedule(static)
#endif
    for (i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;                       /* reduce(+, 0) */
            for (int64_t k = 0; k < K; ++k) {
                double a = (double)A[i * lda + k];
                double b = transB ? (double)B[j * ldb + k] : (double)B[k * ldb + j];
                acc += a * b;                       /* zip, multiply, add */
            }
            C[i * ldc + j] = acc;
        }
    }
    return 0;
}

/*
 * Batched products: for b in [0, batch): C_b = A_b * op(B_b), where
 * X_b = X + b*strideX (element strides).  The paper has no batched product;
 * this is the Section 6.1 definition applied independently to each batch.
 * Threads split the batch loop only.
 */
int oracle_gemm_f32_batched(int64_t batch, int64_t M, int64_t N, int64_t K,
                            const float *A, int64_t lda, int64_t strideA,
                            const float *B, int64_t ldb, int64_t strideB,
                            double *C, int64_t ldc, int64_t strideC,
                            int transB, int nthreads)
{
    if (batch < 0) return -1;
    if (check_args(M, N, K, A, lda, B, ldb, C, ldc, transB) != 0) return -1;
    if (nthreads <= 0) nthreads = 1;
    (void)nthreads;
    int64_t b;
#ifdef _OPENMP
#pragma omp parallel for num_threads(nthreads) schedule(static)
#endif
    for (b = 0; b < batch; ++b) {
        oracle_gemm_f32(M, N, K, A + b * strideA, lda, B + b * strideB, ldb,
                        C + b * strideC, ldc, transB, 1);
    }
    return 0;
}

/*
 * Array packing of B, Section 6.1 (the packedB compute expression):
 *   packedB[x][y][z] = B[y][x*P + z],   shape (ceil(N/P), K, P).
 * The paper fixes P = 32 for its CPU and assumes P divides N; here P is an
 * argument and a ragged last panel is filled with +0.0.
 * Bp must hold ceil(N/P)*K*P floats.  B is read through op(B) as above.
 */
int oracle_pack_b(int64_t N, int64_t K, const float *B, int64_t ldb, int transB,
                  int64_t P, float *Bp)
{
    if (N < 0 || K < 0 || P <= 0) return -1;
    if (transB ? ldb < (K > 1 ? K : 1) : ldb < (N > 1 ? N : 1)) return -1;
    if (N > 0 && K > 0 && (B == NULL || Bp == NULL)) return -1;
    int64_t panels = (N + P - 1) / P;
    for (int64_t x = 0; x < panels; ++x)
        for (int64_t y = 0; y < K; ++y)
            for (int64_t z = 0; z < P; ++z) {
                int64_t col = x * P + z;
                float v = 0.0f;
                if (col < N) v = transB ? B[col * ldb + y] : B[y * ldb + col];
                Bp[(x * K + y) * P + z] = v;
            }
    return 0;
}

/*
 * Product on the packed operand, Section 6.1 (the rewritten compute
 * expression that follows packedB):
 *   C[x][y] = sum_k A[x][k] * packedB[y / P][k][y mod P].
 */
int oracle_gemm_f32_packed(int64_t M, int64_t N, int64_t K,
                           const float *A, int64_t lda,
                           const float *Bp, int64_t P,
                           double *C, int64_t ldc, int nthreads)
{
    if (M < 0 || N < 0 || K < 0 || P <= 0) return -1;
    if (lda < (K > 1 ? K : 1) || ldc < (N > 1 ? N : 1)) return -1;
    if (M > 0 && N > 0 && C == NULL) return -1;
    if (M > 0 && N > 0 && K > 0 && (A == NULL || Bp == NULL)) return -1;
    if (nthreads <= 0) nthreads = 1;
    (void)nthreads;
    int64_t x;
#ifdef _OPENMP
#pragma omp parallel for num_threads(nthreads) schedule(static)
#endif
    for (x = 0; x < M; ++x) {
        for (int64_t y = 0; y < N; ++y) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += (double)A[x * lda + k] * (double)Bp[((y / P) * K + k) * P + (y % P)];
            C[x * ldc + y] = acc;
        }
    }
    return 0;
}

/* Number of threads an OpenMP build will really use for a request of n. */
int oracle_threads_used(int n)
{
    if (n <= 0) n = 1;
#ifdef _OPENMP
    int used = 0;
#pragma omp parallel num_threads(n)
    {
#pragma omp master
        used = omp_get_num_threads();
    }
    return used;
#else
    return 1;
#endif
}
