"""Pins for a matrix-product implementation `gemm(A, B, transB) -> float64 C`.

Each pin checks the implementation against something fixed by the paper's
definition (Section 6.1 / 6.3) or by mathematics, never against the
implementation's own formula.  The same pins are applied to the CPU oracle and,
in test_pins_have_teeth, to deliberately broken implementations: every planted
mistake must trip at least one pin.
"""
from __future__ import annotations

import os

import numpy as np

from paper_2002_02268_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tiny_products.txt")


def load_golden():
    cases = []
    with open(GOLDEN) as f:
        lines = [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]
    i = 0
    while i < len(lines):
        tag, name, M, N, K = lines[i].split()
        assert tag == "case"
        M, N, K = int(M), int(N), int(K)
        i += 1
        rows = [[float(v) for v in lines[i + r].split()] for r in range(M + K + M)]
        i += M + K + M
        A = np.array(rows[:M], dtype=np.float32).reshape(M, K)
        B = np.array(rows[M:M + K], dtype=np.float32).reshape(K, N)
        C = np.array(rows[M + K:], dtype=np.float64).reshape(M, N)
        cases.append((name, A, B, C))
    return cases


def strided(x: np.ndarray, pad: int = 5) -> np.ndarray:
    """Same values in a buffer whose rows are `pad` elements longer (ld = cols + pad);
    the padding holds NaN so reading it shows up in the result."""
    buf = np.full((x.shape[0], x.shape[1] + pad), np.nan, dtype=x.dtype)
    buf[:, : x.shape[1]] = x
    return buf[:, : x.shape[1]]


def int_brute_force(A: np.ndarray, B: np.ndarray) -> np.ndarray:
    """Exact product of integer-valued matrices in Python integers (no floating point)."""
    M, K = A.shape
    N = B.shape[1]
    Ai = [[int(v) for v in row] for row in A]
    Bi = [[int(v) for v in row] for row in B]
    out = np.zeros((M, N), dtype=np.int64)
    for i in range(M):
        for j in range(N):
            s = 0
            for k in range(K):
                s += Ai[i][k] * Bi[k][j]
            out[i, j] = s
    return out


# ----------------------------------------------------------------------------- pins

def pin_golden(gemm):
    for name, A, B, C in load_golden():
        got = gemm(A, B, False)
        assert got.shape == C.shape, name
        assert np.array_equal(got, C), f"golden case {name}: {got} != {C}"
        got_t = gemm(A, np.ascontiguousarray(B.T), True)
        assert np.array_equal(got_t, C), f"golden case {name} (transB)"


def pin_int_brute_force(gemm):
    for seed, (M, N, K) in enumerate([(1, 1, 1), (2, 2, 2), (3, 2, 4), (1, 7, 5), (6, 1, 3), (5, 9, 7)]):
        A = synth.small_ints((M, K), seed + 100, synth.TENSOR_A, -3, 3)
        B = synth.small_ints((K, N), seed + 100, synth.TENSOR_B, -3, 3)
        want = int_brute_force(A, B)
        assert np.array_equal(gemm(A, B, False), want.astype(np.float64))
        assert np.array_equal(gemm(A, np.ascontiguousarray(B.T), True), want.astype(np.float64))


def pin_exact_integer_regime(gemm):
    """Entries in {-2..2}: every partial sum is an integer below 2^24, so the product
    is exact in any order; compare with an int64 library product."""
    for seed, (M, N, K) in enumerate([(37, 29, 53), (64, 64, 64), (33, 70, 130)]):
        A = synth.small_ints((M, K), seed + 200, synth.TENSOR_A)
        B = synth.small_ints((K, N), seed + 200, synth.TENSOR_B)
        want = A.astype(np.int64) @ B.astype(np.int64)
        assert np.array_equal(gemm(A, B, False), want.astype(np.float64))
        assert np.array_equal(gemm(strided(A), strided(B), False), want.astype(np.float64))
        Bt = np.ascontiguousarray(B.T)
        assert np.array_equal(gemm(A, Bt, True), want.astype(np.float64))
        assert np.array_equal(gemm(strided(A), strided(Bt), True), want.astype(np.float64))


def pin_identity(gemm):
    A = synth.uniform((23, 17), 300, synth.TENSOR_A)
    assert np.array_equal(gemm(A, np.eye(17, dtype=np.float32), False), A.astype(np.float64))
    assert np.array_equal(gemm(A, np.eye(17, dtype=np.float32), True), A.astype(np.float64))
    B = synth.uniform((23, 31), 300, synth.TENSOR_B)
    assert np.array_equal(gemm(np.eye(23, dtype=np.float32), B, False), B.astype(np.float64))
    assert np.array_equal(gemm(np.eye(23, dtype=np.float32), np.ascontiguousarray(B.T), True),
                          B.astype(np.float64))


def pin_all_ones(gemm):
    for M, N, K in [(3, 5, 7), (16, 8, 129), (2, 2, 1000)]:
        got = gemm(np.ones((M, K), np.float32), np.ones((K, N), np.float32), False)
        assert np.array_equal(got, np.full((M, N), float(K)))


def pin_indicator(gemm):
    """A = e_i e_k^T picks row k of B into row i of C; B = e_k e_j^T picks column k of A
    into column j of C.  Includes the last row / column / k."""
    M, N, K = 11, 13, 9
    A0 = synth.uniform((M, K), 400, synth.TENSOR_A)
    B0 = synth.uniform((K, N), 400, synth.TENSOR_B)
    for (i, k, j) in [(0, 0, 0), (M - 1, K - 1, N - 1), (3, 7, 2), (10, 0, 12)]:
        A = np.zeros((M, K), np.float32)
        A[i, k] = 1.0
        want = np.zeros((M, N))
        want[i, :] = B0[k, :]
        assert np.array_equal(gemm(A, B0, False), want)
        assert np.array_equal(gemm(A, np.ascontiguousarray(B0.T), True), want)
        B = np.zeros((K, N), np.float32)
        B[k, j] = 1.0
        want = np.zeros((M, N))
        want[:, j] = A0[:, k]
        assert np.array_equal(gemm(A0, B, False), want)
        assert np.array_equal(gemm(A0, np.ascontiguousarray(B.T), True), want)


def pin_transpose(gemm):
    """(AB)^T = B^T A^T, bit-identical when products commute exactly and k runs in the
    same order; and the transB storage flag names the same product."""
    A = synth.uniform((19, 27), 500, synth.TENSOR_A)
    B = synth.uniform((27, 14), 500, synth.TENSOR_B)
    C = gemm(A, B, False)
    Ct = gemm(np.ascontiguousarray(B.T), np.ascontiguousarray(A.T), False)
    assert np.array_equal(C.T, Ct)
    assert np.array_equal(gemm(A, np.ascontiguousarray(B.T), True), C)
    # B^T A^T with A^T handed over as "stored transposed" = A itself
    assert np.array_equal(gemm(np.ascontiguousarray(B.T), A, True), C.T)


def pin_vector_associativity(gemm):
    """A(Bx) = (AB)x, the right-hand side from the implementation's C, the left from two
    fp64 matrix-vector products."""
    A = synth.uniform((40, 300), 600, synth.TENSOR_A)
    B = synth.uniform((300, 50), 600, synth.TENSOR_B)
    x = synth.signs(50, 600)
    C = gemm(A, B, False)
    lhs = A.astype(np.float64) @ (B.astype(np.float64) @ x)
    assert np.max(np.abs(C @ x - lhs)) <= 1e-11


def pin_library_product(gemm):
    """Agreement with a library fp64 product to fp64 rounding (K * 2^-53 * sum|a||b|)."""
    for dist in (synth.uniform, synth.normal):
        A = dist((45, 257), 700, synth.TENSOR_A)
        B = dist((257, 38), 700, synth.TENSOR_B)
        want = A.astype(np.float64) @ B.astype(np.float64)
        bound = 257 * 2.0 ** -53 * (np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64))
        assert np.all(np.abs(gemm(A, B, False) - want) <= bound)
        assert np.all(np.abs(gemm(strided(A), strided(np.ascontiguousarray(B.T)), True) - want) <= bound)


def pin_fp64_accumulation(gemm):
    """A sum that fp32 accumulation gets wrong: 2^24 + 1 + 1 - 2^24 = 2 needs more than
    24 significand bits in the running sum."""
    A = np.array([[16777216.0, 1.0, 1.0, -16777216.0]], dtype=np.float32)
    B = np.ones((4, 1), dtype=np.float32)
    assert gemm(A, B, False)[0, 0] == 2.0


def pin_empty(gemm):
    assert gemm(np.zeros((0, 4), np.float32), np.zeros((4, 3), np.float32), False).shape == (0, 3)
    assert gemm(np.zeros((2, 4), np.float32), np.zeros((4, 0), np.float32), False).shape == (2, 0)
    got = gemm(np.zeros((2, 0), np.float32), np.zeros((0, 3), np.float32), False)
    assert got.shape == (2, 3) and np.array_equal(got, np.zeros((2, 3)))
    assert not np.signbit(got).any()


ALL_PINS = [pin_golden, pin_int_brute_force, pin_exact_integer_regime, pin_identity, pin_all_ones,
            pin_indicator, pin_transpose, pin_vector_associativity, pin_library_product,
            pin_fp64_accumulation, pin_empty]
