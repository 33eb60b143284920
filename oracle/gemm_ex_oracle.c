/*
 * CPU oracle for the general form of the fp32 matrix product:
 *     C = alpha * op(A) * op(B) + beta * C0.
 *
 * TEST INFRASTRUCTURE ONLY: the plain definition the GPU library is checked
 * against; it shares nothing with the GPU path and is never called from it.
 *
 * The paper's product (Section 6.1, the compute expression; Section 6.3, the
 * RISE program mm) is the case alpha = 1, beta = 0, op(A) = A.  Section 6.3
 * reads b through transpose(b) as a view of the caller's array; transA applies
 * the same view to a.  The scaling by alpha and the beta * C0 term are not in
 * the paper; they are the usual library convention layered on its product:
 *     C[i][j] = alpha * ( sum_{k=0}^{K-1} opA[i][k] * opB[k][j] ) + beta * C0[i][j],
 * and for beta == 0 the old contents C0 are not read at all (they may hold NaN),
 * which is what "C is overwritten" means in the paper's own case.
 *
 * Arithmetic: operands, alpha, beta and C0 are binary32 widened to binary64;
 * the sum runs over k ascending in binary64; the two scalings and the final
 * addition are binary64 operations; the result stays binary64.
 *
 * Pinned (tests/test_oracle_ex_pins.py) by exact integer brute force with
 * integer alpha and beta, by the reduction to the plain oracle's bit pattern for
 * alpha = 1, beta = 0, by transposed copies of the same operands, by
 * A = 0 (result beta*C0 exactly), by NaN-filled C0 under beta = 0, by a library
 * matrix product, and by planted mistakes that each trip a pin.
 *
 * Layout (element strides, row-major storage):
 *   transA == 0: A stored M x K, opA[i][k] = A[i*lda + k], lda >= K.
 *   transA != 0: A stored K x M, opA[i][k] = A[k*lda + i], lda >= M.
 *   transB == 0: B stored K x N, opB[k][j] = B[k*ldb + j], ldb >= N.
 *   transB != 0: B stored N x K, opB[k][j] = B[j*ldb + k], ldb >= K.
 *   C0 (float) and C (double) are M x N, ldc0 >= N, ldc >= N.  Elements outside
 *   [0,M) x [0,N) are never written.
 */
#include <stddef.h>
#include <stdint.h>

static int64_t at_least_one(int64_t v) { return v > 1 ? v : 1; }

/* Returns 0 on success, -1 on an invalid dimension / stride / null pointer. */
int oracle_gemm_f32_ex(int64_t M, int64_t N, int64_t K, float alpha,
                       const float *A, int64_t lda, int transA,
                       const float *B, int64_t ldb, int transB,
                       float beta, const float *C0, int64_t ldc0,
                       double *C, int64_t ldc, int nthreads)
{
    if (M < 0 || N < 0 || K < 0) return -1;
    if (lda < at_least_one(transA ? M : K)) return -1;
    if (ldb < at_least_one(transB ? K : N)) return -1;
    if (ldc < at_least_one(N)) return -1;
    if (M > 0 && N > 0 && C == NULL) return -1;
    if (M > 0 && N > 0 && K > 0 && (A == NULL || B == NULL)) return -1;
    if (beta != 0.0f && (ldc0 < at_least_one(N) || (M > 0 && N > 0 && C0 == NULL))) return -1;
    if (nthreads <= 0) nthreads = 1;
    (void)nthreads;
    int64_t i;
#ifdef _OPENMP
#pragma omp parallel for num_threads(nthreads) schedule(static)
#endif
    for (i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double a = transA ? (double)A[k * lda + i] : (double)A[i * lda + k];
                double b = transB ? (double)B[j * ldb + k] : (double)B[k * ldb + j];
                acc += a * b;
            }
            double r = (double)alpha * acc;
            if (beta != 0.0f) r += (double)beta * (double)C0[i * ldc0 + j];
            C[i * ldc + j] = r;
        }
    }
    return 0;
}
