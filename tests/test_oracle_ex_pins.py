"""Pins for the general-form oracle  alpha * op(A) * op(B) + beta * C0.

Every pin compares against something the definition fixes without going through the oracle's own
formula: exact Python-integer brute force, the plain-product oracle's bit pattern in the paper's own
case (alpha = 1, beta = 0, A not transposed; Section 6.1 / 6.3), transposed copies of the operands
(the transpose of Section 6.3 is a view: the values read are the same), degenerate operands, a
library matrix product.  test_ex_pins_have_teeth plants mistakes and requires each to trip a pin."""
from __future__ import annotations

import numpy as np
import pytest

import oracle
from paper_2002_02268_amd import synth

from pins import strided


def stored(X: np.ndarray, trans: bool) -> np.ndarray:
    """The array a caller would hold for logical operand X under the given transpose flag."""
    return np.ascontiguousarray(X.T) if trans else X


def int_brute_force_ex(A, B, C0, alpha, beta):
    M, K = A.shape
    N = B.shape[1]
    out = np.zeros((M, N), dtype=np.int64)
    for i in range(M):
        for j in range(N):
            s = 0
            for k in range(K):
                s += int(A[i, k]) * int(B[k, j])
            out[i, j] = int(alpha) * s + (int(beta) * int(C0[i, j]) if beta != 0 else 0)
    return out


FLAGS = [(False, False), (False, True), (True, False), (True, True)]


def pin_int_brute_force(gemm_ex):
    for seed, (M, N, K) in enumerate([(1, 1, 1), (2, 3, 2), (3, 2, 4), (1, 7, 5), (6, 1, 3), (5, 9, 7), (4, 4, 3)]):
        A = synth.small_ints((M, K), seed + 700, synth.TENSOR_A, -3, 3)
        B = synth.small_ints((K, N), seed + 700, synth.TENSOR_B, -3, 3)
        C0 = synth.small_ints((M, N), seed + 700, 2, -5, 5)
        for alpha, beta in [(1, 0), (2, 0), (1, 1), (-3, 2), (0, 4), (0, 0)]:
            want = int_brute_force_ex(A, B, C0, alpha, beta).astype(np.float64)
            for tA, tB in FLAGS:
                got = gemm_ex(stored(A, tA), stored(B, tB), C0, alpha, beta, tA, tB)
                assert np.array_equal(got, want), (M, N, K, alpha, beta, tA, tB)


def pin_reduces_to_plain_product(gemm_ex):
    """alpha = 1, beta = 0: the paper's product; bit-identical to the plain oracle (same k order)."""
    for seed, (M, N, K) in enumerate([(7, 5, 9), (33, 17, 65), (1, 40, 3)]):
        A = synth.uniform((M, K), seed + 720, synth.TENSOR_A)
        B = synth.uniform((K, N), seed + 720, synth.TENSOR_B)
        plain = oracle.gemm_f32(A, B)
        for tA, tB in FLAGS:
            got = gemm_ex(stored(A, tA), stored(B, tB), None, 1.0, 0.0, tA, tB)
            assert np.array_equal(got, plain), (tA, tB)


def pin_beta_zero_never_reads_c0(gemm_ex):
    A = synth.uniform((6, 4), 730, synth.TENSOR_A)
    B = synth.uniform((4, 5), 730, synth.TENSOR_B)
    poison = np.full((6, 5), np.nan, np.float32)
    got = gemm_ex(A, B, poison, 1.5, 0.0, False, False)
    assert np.isfinite(got).all()
    assert np.array_equal(got, gemm_ex(A, B, None, 1.5, 0.0, False, False))


def pin_zero_a_gives_beta_c0(gemm_ex):
    """A = 0: the result is beta*C0, one exact binary64 product per element."""
    C0 = synth.uniform((5, 8), 740, 2)
    B = synth.uniform((3, 8), 740, synth.TENSOR_B)
    beta = np.float32(0.3)
    got = gemm_ex(np.zeros((5, 3), np.float32), B, C0, 7.0, float(beta), False, False)
    assert np.array_equal(got, np.float64(beta) * C0.astype(np.float64))


def pin_alpha_and_beta_scale_linearly(gemm_ex):
    """Powers of two scale exactly: f(4a, 2b) relates to f(a, b) pieces without rounding."""
    A = synth.uniform((9, 11), 750, synth.TENSOR_A)
    B = synth.uniform((11, 6), 750, synth.TENSOR_B)
    C0 = synth.uniform((9, 6), 750, 2)
    prod = gemm_ex(A, B, None, 1.0, 0.0, False, False)
    assert np.array_equal(gemm_ex(A, B, None, 4.0, 0.0, False, False), 4.0 * prod)
    assert np.array_equal(gemm_ex(A, B, None, -0.5, 0.0, False, False), -0.5 * prod)
    got = gemm_ex(A, B, C0, 1.0, 2.0, False, False)
    assert np.array_equal(got, prod + 2.0 * C0.astype(np.float64))   # one rounding each side, same operands
    # K = 0: the empty sum is 0, so the result is beta*C0 (or 0)
    E = gemm_ex(np.zeros((9, 0), np.float32), np.zeros((0, 6), np.float32), C0, 3.0, 0.5, False, False)
    assert np.array_equal(E, 0.5 * C0.astype(np.float64))


def pin_library_product(gemm_ex):
    A = synth.uniform((40, 70), 760, synth.TENSOR_A)
    B = synth.uniform((70, 30), 760, synth.TENSOR_B)
    C0 = synth.uniform((40, 30), 760, 2)
    alpha, beta = np.float32(1.7), np.float32(-0.6)
    want = np.float64(alpha) * (A.astype(np.float64) @ B.astype(np.float64)) + np.float64(beta) * C0.astype(np.float64)
    for tA, tB in FLAGS:
        got = gemm_ex(stored(A, tA), stored(B, tB), C0, float(alpha), float(beta), tA, tB)
        assert np.max(np.abs(got - want)) <= 1e-12


def pin_row_padding_is_not_read(gemm_ex):
    A = synth.uniform((6, 9), 770, synth.TENSOR_A)
    B = synth.uniform((9, 4), 770, synth.TENSOR_B)
    C0 = synth.uniform((6, 4), 770, 2)
    want = gemm_ex(A, B, C0, 2.0, 3.0, False, False)
    for tA, tB in FLAGS:
        got = gemm_ex(strided(stored(A, tA)), strided(stored(B, tB)), strided(C0), 2.0, 3.0, tA, tB)
        assert np.array_equal(got, want)


ALL_EX_PINS = [pin_int_brute_force, pin_reduces_to_plain_product, pin_beta_zero_never_reads_c0,
               pin_zero_a_gives_beta_c0, pin_alpha_and_beta_scale_linearly, pin_library_product,
               pin_row_padding_is_not_read]


def oracle_ex(A, B, C0, alpha, beta, tA, tB):
    return oracle.gemm_f32_ex(A, B, C0, alpha, beta, tA, tB)


@pytest.mark.parametrize("pin", ALL_EX_PINS, ids=lambda p: p.__name__)
def test_oracle_ex_pin(pin):
    pin(oracle_ex)


def test_oracle_ex_threads_do_not_change_result():
    A = synth.uniform((37, 50), 780, synth.TENSOR_A)
    B = synth.uniform((50, 21), 780, synth.TENSOR_B)
    C0 = synth.uniform((37, 21), 780, 2)
    one = oracle.gemm_f32_ex(A, B, C0, 1.25, 0.75, nthreads=1)
    assert np.array_equal(one, oracle.gemm_f32_ex(A, B, C0, 1.25, 0.75, nthreads=4))


def test_oracle_ex_rejects_bad_arguments():
    A = np.zeros((4, 3), np.float32)
    B = np.zeros((3, 5), np.float32)
    with pytest.raises(ValueError):
        oracle.gemm_f32_ex(A, B, None, 1.0, 1.0)          # beta != 0 without C0
    with pytest.raises(ValueError):
        oracle.gemm_f32_ex(A, B, transA=True)            # inner dimensions differ
    with pytest.raises(ValueError):
        oracle.gemm_f32_ex(A, B, np.zeros((4, 4), np.float32), 1.0, 1.0)


# ------------------------------------------------------------------ planted mistakes

def _logical(A, B, tA, tB):
    A = A.astype(np.float64)
    B = B.astype(np.float64)
    return (A.T if tA else A), (B.T if tB else B)


def _finish(P, C0, alpha, beta):
    r = np.float64(np.float32(alpha)) * P
    if beta != 0:
        r = r + np.float64(np.float32(beta)) * C0.astype(np.float64)
    return r


def mutant_ignores_transa(A, B, C0, alpha, beta, tA, tB):
    Al, Bl = _logical(A, B, False if A.shape[0] == A.shape[1] else tA, tB)
    return _finish(Al @ Bl, C0, alpha, beta)


def mutant_alpha_on_c0(A, B, C0, alpha, beta, tA, tB):
    Al, Bl = _logical(A, B, tA, tB)
    P = Al @ Bl
    return np.float64(alpha) * (P + (np.float64(np.float32(beta)) * C0.astype(np.float64) if beta != 0 else 0.0))


def mutant_beta_ignored(A, B, C0, alpha, beta, tA, tB):
    Al, Bl = _logical(A, B, tA, tB)
    return _finish(Al @ Bl, C0, alpha, 0.0)


def mutant_alpha_ignored(A, B, C0, alpha, beta, tA, tB):
    Al, Bl = _logical(A, B, tA, tB)
    return _finish(Al @ Bl, C0, 1.0, beta)


def mutant_reads_c0_when_beta_zero(A, B, C0, alpha, beta, tA, tB):
    Al, Bl = _logical(A, B, tA, tB)
    r = np.float64(np.float32(alpha)) * (Al @ Bl)
    if C0 is not None:
        r = r + np.float64(np.float32(beta)) * C0.astype(np.float64)
    return r


def mutant_swapped_scalars(A, B, C0, alpha, beta, tA, tB):
    Al, Bl = _logical(A, B, tA, tB)
    if beta == 0:
        return _finish(Al @ Bl, C0, alpha, beta)
    return _finish(Al @ Bl, C0, beta, alpha)


def mutant_c0_transposed(A, B, C0, alpha, beta, tA, tB):
    Al, Bl = _logical(A, B, tA, tB)
    if beta != 0 and C0.shape[0] == C0.shape[1]:
        C0 = C0.T
    return _finish(Al @ Bl, C0, alpha, beta)


def mutant_float32_scaling(A, B, C0, alpha, beta, tA, tB):
    Al, Bl = _logical(A, B, tA, tB)
    P = (Al @ Bl).astype(np.float32)
    r = np.float32(alpha) * P
    if beta != 0:
        r = r + np.float32(beta) * C0
    return r.astype(np.float64)


def mutant_reads_padding_of_transposed_a(A, B, C0, alpha, beta, tA, tB):
    Am = A
    if tA and A.shape[0] > 1 and A.strides[0] != 4 * A.shape[1]:
        flat = np.lib.stride_tricks.as_strided(A, shape=(A.shape[0] * A.shape[1],), strides=(4,))
        Am = flat.reshape(A.shape)
    Al, Bl = _logical(Am, B, tA, tB)
    return _finish(Al @ Bl, C0, alpha, beta)


EX_MUTANTS = [mutant_ignores_transa, mutant_alpha_on_c0, mutant_beta_ignored, mutant_alpha_ignored,
              mutant_reads_c0_when_beta_zero, mutant_swapped_scalars, mutant_c0_transposed,
              mutant_float32_scaling, mutant_reads_padding_of_transposed_a]


@pytest.mark.parametrize("mutant", EX_MUTANTS, ids=lambda m: m.__name__)
def test_ex_pins_have_teeth(mutant):
    tripped = []
    for pin in ALL_EX_PINS:
        try:
            pin(mutant)
        except AssertionError:
            tripped.append(pin.__name__)
    assert tripped, f"{mutant.__name__} passes every pin"
