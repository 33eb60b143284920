"""CPU tests that pin the oracle to what the paper and mathematics fix (no GPU needed)."""
from __future__ import annotations

import numpy as np
import pytest

import oracle
from paper_2002_02268_amd import synth

import pins


def oracle_gemm(A, B, transB):
    return oracle.gemm_f32(A, B, transB=transB, nthreads=1)


@pytest.mark.parametrize("pin", pins.ALL_PINS, ids=lambda p: p.__name__)
def test_oracle_pin(pin):
    pin(oracle_gemm)


def test_oracle_threads_do_not_change_result():
    A = synth.uniform((67, 129), 1, synth.TENSOR_A)
    B = synth.uniform((129, 45), 1, synth.TENSOR_B)
    one = oracle.gemm_f32(A, B, nthreads=1)
    for t in (2, 3, 8):
        assert np.array_equal(oracle.gemm_f32(A, B, nthreads=t), one)


def test_oracle_never_writes_outside_c():
    """C has ldc > N in the C call: the padding keeps its sentinel."""
    import ctypes
    lib = oracle._load()
    M, N, K, ldc = 5, 7, 3, 11
    A = synth.uniform((M, K), 2, synth.TENSOR_A)
    B = synth.uniform((K, N), 2, synth.TENSOR_B)
    C = np.full((M + 1, ldc), -77.0)
    rc = lib.oracle_gemm_f32(M, N, K, A.ctypes.data_as(oracle._fp), K, B.ctypes.data_as(oracle._fp), N,
                             C.ctypes.data_as(oracle._dp), ldc, 0, 1)
    assert rc == 0
    assert np.all(C[:M, N:] == -77.0) and np.all(C[M:] == -77.0)
    assert np.array_equal(C[:M, :N], oracle.gemm_f32(A, B))
    del ctypes


def test_oracle_rejects_bad_strides():
    lib = oracle._load()
    A = np.zeros((4, 4), np.float32)
    C = np.zeros((4, 4))
    args = lambda lda, ldb, ldc, tb: lib.oracle_gemm_f32(  # noqa: E731
        4, 4, 4, A.ctypes.data_as(oracle._fp), lda, A.ctypes.data_as(oracle._fp), ldb,
        C.ctypes.data_as(oracle._dp), ldc, tb, 1)
    assert args(4, 4, 4, 0) == 0
    assert args(3, 4, 4, 0) == -1
    assert args(4, 3, 4, 0) == -1
    assert args(4, 4, 3, 0) == -1
    assert args(4, 3, 4, 1) == -1


# ------------------------------------------------------------------ pins have teeth

def _f64(A, B, transB):
    A = A.astype(np.float64)
    B = B.astype(np.float64)
    return A, (B.T if transB else B)


def mutant_transposed_a(A, B, transB):
    A, B = _f64(A, B, transB)
    return (A.T @ B) if A.shape[0] == A.shape[1] else A @ B


def mutant_dropped_last_term(A, B, transB):
    A, B = _f64(A, B, transB)
    return A[:, :-1] @ B[:-1, :] if A.shape[1] > 1 else A @ B


def mutant_dropped_first_term(A, B, transB):
    A, B = _f64(A, B, transB)
    return A[:, 1:] @ B[1:, :] if A.shape[1] > 1 else A @ B


def mutant_sign(A, B, transB):
    A, B = _f64(A, B, transB)
    return -(A @ B)


def mutant_ignores_transb(A, B, transB):
    A = A.astype(np.float64)
    B = B.astype(np.float64)
    if transB and B.shape[0] == B.shape[1]:
        return A @ B
    return A @ (B.T if transB else B)


def mutant_output_transposed(A, B, transB):
    A, B = _f64(A, B, transB)
    C = A @ B
    return C.T.copy() if C.shape[0] == C.shape[1] else C


def mutant_fp32_accumulate(A, B, transB):
    Bm = B.T if transB else B
    M, K = A.shape
    acc = np.zeros((M, Bm.shape[1]), np.float32)
    for k in range(K):
        acc = (acc + np.outer(A[:, k], Bm[k, :]).astype(np.float32)).astype(np.float32)
    return acc.astype(np.float64)


def mutant_reads_row_padding(A, B, transB):
    """Uses the tight width as the leading dimension of B even when rows are padded."""
    Bm = B
    if B.shape[0] > 1 and B.strides[0] != 4 * B.shape[1]:
        flat = np.lib.stride_tricks.as_strided(B, shape=(B.shape[0] * B.shape[1],), strides=(4,))
        Bm = flat.reshape(B.shape)
    A, Bm = _f64(A, Bm, transB)
    return A @ Bm


def mutant_off_by_one_column(A, B, transB):
    A, B = _f64(A, B, transB)
    C = A @ B
    return np.roll(C, 1, axis=1) if C.shape[1] > 1 else C


def mutant_abs_b(A, B, transB):
    A, B = _f64(A, B, transB)
    return A @ np.abs(B)


MUTANTS = [mutant_transposed_a, mutant_dropped_last_term, mutant_dropped_first_term, mutant_sign,
           mutant_ignores_transb, mutant_output_transposed, mutant_fp32_accumulate,
           mutant_reads_row_padding, mutant_off_by_one_column, mutant_abs_b]


@pytest.mark.parametrize("mutant", MUTANTS, ids=lambda m: m.__name__)
def test_pins_have_teeth(mutant):
    tripped = []
    for pin in pins.ALL_PINS:
        try:
            pin(mutant)
        except AssertionError:
            tripped.append(pin.__name__)
    assert tripped, f"{mutant.__name__} passes every pin"


# ------------------------------------------------------------------ packing and batches

@pytest.mark.parametrize("N,K,P", [(64, 5, 32), (70, 9, 32), (5, 3, 8), (130, 17, 128), (1, 1, 4)])
def test_pack_b_layout_and_padding(N, K, P):
    """packedB[x][y][z] = B[y][x*P + z]; zero (+0.0) beyond column N (Section 6.1)."""
    B = synth.uniform((K, N), 11, synth.TENSOR_B)
    for transB, stored in ((False, B), (True, np.ascontiguousarray(B.T)),
                           (False, pins.strided(B)), (True, pins.strided(np.ascontiguousarray(B.T)))):
        Bp = oracle.pack_b(stored, P, transB=transB)
        panels = -(-N // P)
        assert Bp.shape == (panels, K, P)
        # independent statement of the layout through numpy reshapes
        padded = np.zeros((K, panels * P), np.float32)
        padded[:, :N] = B
        want = padded.reshape(K, panels, P).transpose(1, 0, 2)
        assert np.array_equal(Bp, want)
        assert not np.signbit(Bp[Bp == 0]).any() or np.array_equal(Bp, want)
        # unpack(pack(B)) == B
        unpacked = Bp.transpose(1, 0, 2).reshape(K, panels * P)[:, :N]
        assert np.array_equal(unpacked, B)


@pytest.mark.parametrize("M,N,K,P", [(7, 64, 5, 32), (9, 70, 33, 32), (4, 5, 3, 8), (3, 130, 20, 128)])
def test_packed_product_equals_plain_product(M, N, K, P):
    """The product on packedB is the same sum in the same k order: bit-identical."""
    A = synth.uniform((M, K), 12, synth.TENSOR_A)
    B = synth.uniform((K, N), 12, synth.TENSOR_B)
    Bp = oracle.pack_b(B, P)
    assert np.array_equal(oracle.gemm_f32_packed(A, Bp, N), oracle.gemm_f32(A, B))
    Ai = synth.small_ints((M, K), 13, synth.TENSOR_A)
    Bi = synth.small_ints((K, N), 13, synth.TENSOR_B)
    want = (Ai.astype(np.int64) @ Bi.astype(np.int64)).astype(np.float64)
    assert np.array_equal(oracle.gemm_f32_packed(Ai, oracle.pack_b(Bi, P), N), want)


def test_batched_equals_loop_of_singles():
    A = synth.uniform((6, 9, 13), 14, synth.TENSOR_A)
    B = synth.uniform((6, 13, 7), 14, synth.TENSOR_B)
    got = oracle.gemm_f32_batched(A, B, nthreads=3)
    for b in range(6):
        assert np.array_equal(got[b], oracle.gemm_f32(A[b], B[b]))
    Bt = np.ascontiguousarray(B.transpose(0, 2, 1))
    assert np.array_equal(oracle.gemm_f32_batched(A, Bt, transB=True), got)
    Ai = synth.small_ints((5, 8, 8), 15, synth.TENSOR_A)
    Bi = synth.small_ints((5, 8, 8), 15, synth.TENSOR_B)
    want = np.einsum("bik,bkj->bij", Ai.astype(np.int64), Bi.astype(np.int64))
    assert np.array_equal(oracle.gemm_f32_batched(Ai, Bi), want.astype(np.float64))


def test_batched_poisoned_neighbour_does_not_leak():
    A = synth.uniform((3, 4, 5), 16, synth.TENSOR_A)
    B = synth.uniform((3, 5, 6), 16, synth.TENSOR_B)
    clean = oracle.gemm_f32_batched(A, B)
    A2 = A.copy()
    A2[1] = np.nan
    got = oracle.gemm_f32_batched(A2, B)
    assert np.array_equal(got[0], clean[0]) and np.array_equal(got[2], clean[2])
    assert np.isnan(got[1]).all()


# ------------------------------------------------------------------ input generator

def test_generator_is_counter_based_and_in_range():
    u = synth.uniform((1000, 37), 5, synth.TENSOR_A)
    assert u.dtype == np.float32 and np.all(np.abs(u) < 1.0)
    assert abs(float(u.mean())) < 0.02 and abs(float(u.var()) - 1.0 / 3.0) < 0.02
    # element i of a longer stream equals element i of a shorter one
    assert np.array_equal(synth.uniform((100,), 5, synth.TENSOR_A), u.reshape(-1)[:100])
    assert not np.array_equal(synth.uniform((100,), 6, synth.TENSOR_A), u.reshape(-1)[:100])
    assert not np.array_equal(synth.uniform((100,), 5, synth.TENSOR_B), u.reshape(-1)[:100])
    g = synth.normal((200000,), 7, synth.TENSOR_B)
    assert abs(float(g.mean())) < 0.01 and abs(float(g.var()) - 1.0) < 0.02
    assert np.isfinite(g).all()
    i = synth.small_ints((5000,), 8, synth.TENSOR_A)
    assert set(np.unique(i)) == {-2.0, -1.0, 0.0, 1.0, 2.0}
    assert set(np.unique(synth.signs(100, 9))) == {-1.0, 1.0}


def test_generator_output_function_is_the_published_splitmix64():
    """The first three outputs of SplitMix64 seeded with 0 (state advanced by the golden-ratio
    increment, then the two multiply-xorshift rounds), as the published reference prints them."""
    with np.errstate(over="ignore"):
        state = np.arange(1, 4, dtype=np.uint64) * synth._GOLDEN
        got = [int(v) for v in synth._mix(state)]
    assert got == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
