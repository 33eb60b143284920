"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Bit-exact where the arithmetic is exact (integer-valued operands, identity,
indicator probes, packing); otherwise max|C - C_ref| <= 1e-3*sqrt(K/1024) (x3 for N(0,1)
operands, whose products have 9x the variance of U(-1,1) ones) and relative Frobenius
error <= 1e-5."""
from __future__ import annotations

import math
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
import workload_refs  # noqa: E402
from paper_2002_02268_amd import binding, synth  # noqa: E402

NTHREADS = min(16, os.cpu_count() or 1)
TILES = {"t256": "0", "t128": "1", "t64": "2", "tb64": "3", "t256x128": "4", "t128x256": "5", "t128x64": "6",
         "t64x128": "7", "t128x32": "8", "t32x128": "9", "tq32": "10", "tq64x32": "11", "tq32x64": "12"}
TILE_DIMS = {"t256": (256, 256), "t128": (128, 128), "t64": (64, 64), "tb64": (64, 64), "t256x128": (256, 128),
             "t128x256": (128, 256), "t128x64": (128, 64), "t64x128": (64, 128),
             "t128x32": (128, 32), "t32x128": (32, 128), "tq32": (32, 32), "tq64x32": (64, 32), "tq32x64": (32, 64)}


def dev(x: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def padded_dev(x: np.ndarray, pad, fill=float("nan")):
    """Device buffer with rows `pad` elements longer than x ("align4": padded so that the row
    length is a multiple of 4 and at least 4 longer); returns (view, whole buffer)."""
    if pad == "align4":
        pad = (-x.shape[1]) % 4 + 4
    buf = torch.full((x.shape[0], x.shape[1] + pad), fill, dtype=torch.float32, device="cuda")
    view = buf[:, : x.shape[1]]
    view.copy_(torch.from_numpy(np.ascontiguousarray(x)))
    return view, buf


def check_close(C: np.ndarray, ref: np.ndarray, K: int, scale: float = 1.0):
    assert C.shape == ref.shape
    assert np.isfinite(C).all()
    diff = np.abs(C.astype(np.float64) - ref)
    tol = scale * 1e-3 * math.sqrt(max(K, 1) / 1024.0)
    assert diff.max(initial=0.0) <= tol, f"max abs err {diff.max()} > {tol}"
    denom = np.linalg.norm(ref)
    if denom > 0:
        rel = np.linalg.norm(diff) / denom
        assert rel <= 1e-5, f"relative Frobenius error {rel}"


@pytest.fixture
def force_tile():
    def _set(name):
        if name is None:
            binding.set_test_hooks(force_tile=None)
        else:
            binding.set_test_hooks(force_tile=TILES[name])
    yield _set
    binding.set_test_hooks()


SMALL_SHAPES = [(1, 1, 1), (33, 65, 17), (64, 64, 64), (130, 257, 70), (300, 513, 129), (257, 130, 1), (5, 700, 33)]


@pytest.mark.parametrize("tile", list(TILES))
@pytest.mark.parametrize("transB", [False, True])
@pytest.mark.parametrize("pad", [0, 5, "align4"])
def test_small_shapes_every_tile(force_tile, tile, transB, pad):
    """Several tiles plus ragged tails in M, N and K; tight, odd (ld = dim+5, per-element path)
    and 16-byte-friendly (ld rounded up to a multiple of 4: vector path with ragged edges)
    strides; NaN in all padding and in old C."""
    force_tile(tile)
    for idx, (M, N, K) in enumerate(SMALL_SHAPES):
        print(f"case tile={tile} transB={transB} pad={pad} M={M} N={N} K={K}", flush=True)
        A = synth.uniform((M, K), 20 + idx, synth.TENSOR_A)
        B = synth.uniform((N, K) if transB else (K, N), 20 + idx, synth.TENSOR_B)
        ref = oracle.gemm_f32(A, B, transB=transB, nthreads=NTHREADS)
        dA, _ = padded_dev(A, pad)
        dB, _ = padded_dev(B, pad)
        dC, bufC = padded_dev(np.full((M, N), np.nan, np.float32), pad)
        binding.gemm_f32(dA, dB, dC, transB=transB)
        torch.cuda.synchronize()
        whole = bufC.cpu().numpy()
        check_close(whole[:, :N], ref, K)
        assert np.isnan(whole[:, N:]).all(), "ldc padding was written"


@pytest.mark.parametrize("tile", list(TILES))
@pytest.mark.parametrize("transB", [False, True])
def test_tile_boundary_sweep_bit_exact(force_tile, tile, transB):
    """M and N one below, at, one above and well past a tile boundary, in every combination: edge
    tiles shorter than a tile (masked loads) and edge tiles of longer matrices (moved back inside,
    storing only their own rows and columns).  Integer operands, so every result is exact; C is
    pre-filled with NaN and carries NaN padding that must survive."""
    force_tile(tile)
    BM, BN = TILE_DIMS[tile]
    K = 37
    for M in (BM - 1, BM, BM + 1, 2 * BM + 7):
        for N in (BN - 1, BN, BN + 1, 2 * BN + 9):
            print(f"case tile={tile} transB={transB} M={M} N={N}", flush=True)
            A = synth.small_ints((M, K), 300 + M, synth.TENSOR_A)
            B = synth.small_ints((N, K) if transB else (K, N), 300 + N, synth.TENSOR_B)
            ref = oracle.gemm_f32(A, B, transB=transB, nthreads=NTHREADS)
            dC, bufC = padded_dev(np.full((M, N), np.nan, np.float32), 3)
            binding.gemm_f32(dev(A), dev(B), dC, transB=transB)
            whole = bufC.cpu().numpy()
            assert np.array_equal(whole[:, :N].astype(np.float64), ref)
            assert np.isnan(whole[:, N:]).all()
            # the packed form of the same operand
            Bp = torch.full((binding.pack_b_size(N, K) // 4,), float("nan"), device="cuda")
            binding.pack_b(dev(B), Bp, transB=transB)
            dC2 = torch.full((M, N), float("nan"), device="cuda")
            binding.gemm_f32_packed(dev(A), Bp, dC2)
            assert np.array_equal(dC2.cpu().numpy().astype(np.float64), ref)


@pytest.mark.parametrize("tile", list(TILES))
@pytest.mark.parametrize("transB", [False, True])
def test_integer_operands_bit_exact(force_tile, tile, transB):
    """Entries in {-2..2}: all partial sums are integers below 2^24, exact in any order."""
    force_tile(tile)
    for idx, (M, N, K) in enumerate([(100, 90, 300), (257, 513, 65), (64, 64, 64)]):
        A = synth.small_ints((M, K), 40 + idx, synth.TENSOR_A)
        B = synth.small_ints((N, K) if transB else (K, N), 40 + idx, synth.TENSOR_B)
        ref = oracle.gemm_f32(A, B, transB=transB, nthreads=NTHREADS)
        dC = torch.full((M, N), float("nan"), device="cuda")
        binding.gemm_f32(dev(A), dev(B), dC, transB=transB)
        assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)


def test_identity_and_indicator_probes_bit_exact(force_tile):
    for tile in TILES:
        force_tile(tile)
        M, N, K = 150, 140, 131
        A = synth.uniform((M, K), 50, synth.TENSOR_A)
        dC = torch.empty((M, K), device="cuda")
        binding.gemm_f32(dev(A), dev(np.eye(K, dtype=np.float32)), dC)
        assert np.array_equal(dC.cpu().numpy(), A)
        binding.gemm_f32(dev(A), dev(np.eye(K, dtype=np.float32)), dC, transB=True)
        assert np.array_equal(dC.cpu().numpy(), A)
        B = synth.uniform((K, N), 50, synth.TENSOR_B)
        for (i, k) in [(0, 0), (M - 1, K - 1), (77, 129), (149, 3)]:
            E = np.zeros((M, K), np.float32)
            E[i, k] = 1.0
            dC = torch.full((M, N), float("nan"), device="cuda")
            binding.gemm_f32(dev(E), dev(B), dC)
            want = np.zeros((M, N), np.float32)
            want[i] = B[k]
            assert np.array_equal(dC.cpu().numpy(), want)
            binding.gemm_f32(dev(E), dev(B.T), dC, transB=True)
            assert np.array_equal(dC.cpu().numpy(), want)


def test_all_ones_closed_form():
    for (M, N, K) in [(70, 300, 1000), (256, 256, 4096)]:
        dC = torch.empty((M, N), device="cuda")
        binding.gemm_f32(torch.ones((M, K), device="cuda"), torch.ones((K, N), device="cuda"), dC)
        assert torch.equal(dC, torch.full((M, N), float(K), device="cuda"))


def test_masked_lanes_contribute_exact_zeros():
    """Operands sit inside larger NaN / Inf-filled buffers; tails in M, N and K are all ragged."""
    M, N, K = 131, 77, 45
    A = synth.uniform((M, K), 60, synth.TENSOR_A)
    B = synth.uniform((K, N), 60, synth.TENSOR_B)
    ref = oracle.gemm_f32(A, B)
    for fill in (float("nan"), float("inf")):
        bigA = torch.full((M + 40, K + 40), fill, device="cuda")
        bigB = torch.full((K + 40, N + 40), fill, device="cuda")
        bigA[:M, :K] = dev(A)
        bigB[:K, :N] = dev(B)
        dC = torch.empty((M, N), device="cuda")
        binding.gemm_f32(bigA[:M, :K], bigB[:K, :N], dC)
        check_close(dC.cpu().numpy(), ref, K)


def test_nan_in_range_propagates_only_to_its_row_and_column():
    M, N, K = 70, 90, 40
    A = synth.uniform((M, K), 61, synth.TENSOR_A)
    B = synth.uniform((K, N), 61, synth.TENSOR_B)
    A[13, 7] = np.nan
    dC = torch.empty((M, N), device="cuda")
    binding.gemm_f32(dev(A), dev(B), dC)
    C = dC.cpu().numpy()
    assert np.isnan(C[13]).all() and np.isfinite(np.delete(C, 13, axis=0)).all()


def test_empty_dimensions():
    dA = torch.empty((0, 8), device="cuda")
    dB = torch.empty((8, 5), device="cuda")
    binding.gemm_f32(dA, dB, torch.empty((0, 5), device="cuda"))
    binding.gemm_f32(torch.empty((4, 8), device="cuda"), torch.empty((8, 0), device="cuda"),
                     torch.empty((4, 0), device="cuda"))
    dC = torch.full((37, 41), float("nan"), device="cuda")
    binding.gemm_f32(torch.empty((37, 0), device="cuda"), torch.empty((0, 41), device="cuda"), dC)
    C = dC.cpu().numpy()
    assert np.array_equal(C, np.zeros((37, 41), np.float32)) and not np.signbit(C).any()
    binding.gemm_f32_batched(torch.empty((0, 4, 4), device="cuda"), torch.empty((0, 4, 4), device="cuda"),
                             torch.empty((0, 4, 4), device="cuda"))


def test_error_codes():
    lib = binding.lib()
    buf = torch.zeros(64 * 64, device="cuda")
    other = torch.zeros(64 * 64, device="cuda")
    out = torch.zeros(64 * 64, device="cuda")
    a, b, c = buf.data_ptr(), other.data_ptr(), out.data_ptr()
    assert lib.gemm_f32(8, 8, 8, a, 8, b, 8, c, 8, 0) == 0
    assert lib.gemm_f32(-1, 8, 8, a, 8, b, 8, c, 8, 0) == -1
    assert lib.gemm_f32(8, 8, 8, a, 7, b, 8, c, 8, 0) == -1
    assert lib.gemm_f32(8, 9, 8, a, 8, b, 8, c, 9, 0) == -1      # ldb < N
    assert lib.gemm_f32(8, 9, 4, a, 4, b, 8, c, 9, 1) == 0       # transB: ldb >= K is enough
    assert lib.gemm_f32(8, 8, 8, a, 8, b, 8, c, 7, 0) == -1
    assert lib.gemm_f32(8, 8, 8, a, 8, b, 8, c, 8, 2) == -1
    assert lib.gemm_f32(8, 8, 8, None, 8, b, 8, c, 8, 0) == -2
    assert lib.gemm_f32(8, 8, 8, a, 8, b, 8, None, 8, 0) == -2
    assert lib.gemm_f32(8, 8, 8, a, 8, b, 8, a, 8, 0) == -3
    assert lib.gemm_f32(8, 8, 8, a, 8, b, 8, b, 8, 0) == -3
    assert lib.gemm_f32(1 << 31, 8, 8, a, 8, b, 8, c, 8, 0) == -1
    assert lib.pack_b(8, 8, a, 7, 0, c) == -1
    assert lib.pack_b(8, 8, a, 8, 0, c + 4) == -1
    assert lib.gemm_f32_strerror(-3).decode().startswith("output aliases")
    torch.cuda.synchronize()


def test_run_to_run_bitwise_determinism():
    A, B = synth.make_operands("ragged")
    dA, dB = dev(A), dev(B)
    outs = []
    for _ in range(3):
        dC = torch.empty((1000, 1030), device="cuda")
        binding.gemm_f32(dA, dB, dC)
        outs.append(dC.cpu().numpy())
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


def test_transpose_identity_on_gpu():
    """(AB)^T = B^T A^T and the transB flag: same product within tolerance."""
    A = synth.uniform((210, 330), 62, synth.TENSOR_A)
    B = synth.uniform((330, 190), 62, synth.TENSOR_B)
    ref = oracle.gemm_f32(A, B, nthreads=NTHREADS)
    dC = torch.empty((210, 190), device="cuda")
    binding.gemm_f32(dev(A), dev(B), dC)
    check_close(dC.cpu().numpy(), ref, 330)
    dCt = torch.empty((190, 210), device="cuda")
    binding.gemm_f32(dev(B.T), dev(A.T), dCt)
    check_close(dCt.cpu().numpy().T, ref, 330)
    binding.gemm_f32(dev(B.T), dev(A), dCt, transB=True)
    check_close(dCt.cpu().numpy().T, ref, 330)


# --------------------------------------------------------------------- the five workloads

def test_workload_square1024_full_oracle():
    A, B = workload_refs.operands("square1024")
    dC = torch.full((1024, 1024), float("nan"), device="cuda")
    binding.gemm_f32(dev(A), dev(B), dC)
    check_close(dC.cpu().numpy(), workload_refs.reference("square1024"), 1024)


def test_workload_ragged_full_oracle_with_guards():
    A, B = synth.make_operands("ragged")
    ref = oracle.gemm_f32(A, B, nthreads=NTHREADS)
    guard = torch.full((1000 + 2, 1030), float("nan"), device="cuda")   # one guard row each side
    dC = guard[1:1001]
    binding.gemm_f32(dev(A), dev(B), dC)
    whole = guard.cpu().numpy()
    check_close(whole[1:1001], ref, 999)
    assert np.isnan(whole[0]).all() and np.isnan(whole[1001]).all()


def test_workload_ragged_integer_bit_exact():
    A, B = synth.make_operands("ragged", dist="ints")
    ref = oracle.gemm_f32(A, B, nthreads=NTHREADS)
    dC = torch.empty((1000, 1030), device="cuda")
    binding.gemm_f32(dev(A), dev(B), dC)
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)


def _vector_check(A, B, C, transB, K, seed, scale=1.0):
    """A(Bx) = Cx over the whole output, both sides in fp64 on the host: O(n^2), independent of the
    O(n^3) oracle."""
    N = C.shape[1]
    x = synth.signs(N, seed)
    Bx = (B.astype(np.float64).T @ x) if transB else (B.astype(np.float64) @ x)
    lhs = A.astype(np.float64) @ Bx
    tol = scale * 1e-3 * math.sqrt(K / 1024.0) * math.sqrt(N)
    assert np.max(np.abs(C.astype(np.float64) @ x - lhs)) <= tol


def test_workload_square4096_full_oracle():
    """Every element of the 4096 x 4096 output against the fp64 triple loop (about 22 s of oracle time),
    launched as the benchmark launches it; the tolerance is the one stated over the whole output."""
    A, B = workload_refs.operands("square4096")
    assert binding.variant_name(4096, 4096, 4096) == "t128x128x16/nn/a16"
    dC = torch.full((4096, 4096), float("nan"), device="cuda")
    binding.gemm_f32(dev(A), dev(B), dC)
    C = dC.cpu().numpy()
    check_close(C, workload_refs.reference("square4096"), 4096)
    _vector_check(A, B, C, False, 4096, seed=2)
    # and the same output through the 256 x 256 tile, one tile per compute unit (what products whose operands
    # no longer fit the memory-side cache take)
    binding.set_test_hooks(force_tile=0)
    try:
        assert binding.variant_name(4096, 4096, 4096) == "t256x256x16/nn/a16"
        dC.fill_(float("nan"))
        binding.gemm_f32(dev(A), dev(B), dC)
        check_close(dC.cpu().numpy(), workload_refs.reference("square4096"), 4096)
    finally:
        binding.set_test_hooks()


@pytest.mark.parametrize("name", ["skinny8192", "wide8192"])
def test_workload_one_short_dimension_full_oracle(name):
    """8192 x 32 x 8192 and 32 x 8192 x 8192 (B stored N x K) as the benchmark launches them: every
    element against the oracle, on U(-1,1) and exactly on integer-valued operands."""
    w = synth.WORKLOADS[name]
    assert binding.variant_name(w["M"], w["N"], w["K"], transB=w["transB"]).startswith("t32x32x64k4")
    for dist in (None, "ints"):
        A, B = synth.make_operands(name, dist=dist)
        dC = torch.full((w["M"], w["N"]), float("nan"), device="cuda")
        binding.gemm_f32(dev(A), dev(B), dC, transB=w["transB"])
        C = dC.cpu().numpy()
        ref = oracle.gemm_f32(A, B, transB=w["transB"], nthreads=NTHREADS)
        if dist == "ints":
            assert np.array_equal(C.astype(np.float64), ref)
        else:
            check_close(C, ref, w["K"])


def test_workload_square4096_integer_bit_exact_full_oracle():
    """Whole 4096^2 output, exact: integer-valued operands against the oracle on every row, and the
    +-1 vector check (exact in fp64) over everything."""
    A, B = workload_refs.operands("square4096", "ints")
    dC = torch.empty((4096, 4096), device="cuda")
    binding.gemm_f32(dev(A), dev(B), dC)
    C = dC.cpu().numpy()
    assert np.array_equal(C.astype(np.float64), workload_refs.reference("square4096", "ints"))
    x = synth.signs(4096, 2)
    assert np.array_equal(C.astype(np.float64) @ x, A.astype(np.float64) @ (B.astype(np.float64) @ x))


def test_workload_transb2048_and_packed_full_oracle():
    """2048^3 with B stored N x K, N(0,1) operands, and the same product through pack_b: every element
    of both outputs against the oracle (the plain one, and the one that reads packedB); then the same
    on integer-valued operands, bit for bit."""
    A, Bt = workload_refs.operands("transb2048")          # Bt is B stored N x K
    ref = workload_refs.reference("transb2048")
    dA, dBt = dev(A), dev(Bt)
    dC = torch.full((2048, 2048), float("nan"), device="cuda")
    binding.gemm_f32(dA, dBt, dC, transB=True)
    C = dC.cpu().numpy()
    check_close(C, ref, 2048, 3.0)
    _vector_check(A, Bt, C, True, 2048, seed=3, scale=3.0)

    P = binding.pack_b_panel_width()
    nbytes = binding.pack_b_size(2048, 2048)
    assert nbytes == (2048 // P) * 2048 * P * 4
    dBp = torch.full((nbytes // 4,), float("nan"), device="cuda")
    binding.pack_b(dBt, dBp, transB=True)
    want = oracle.pack_b(Bt, P, transB=True)
    assert np.array_equal(dBp.cpu().numpy().reshape(want.shape), want)
    dC2 = torch.full((2048, 2048), float("nan"), device="cuda")
    binding.gemm_f32_packed(dA, dBp, dC2)
    C2 = dC2.cpu().numpy()
    ref_packed = oracle.gemm_f32_packed(A, want, 2048, nthreads=NTHREADS)
    assert np.array_equal(ref_packed, ref)                 # the rewritten expression names the same sums
    check_close(C2, ref_packed, 2048, 3.0)
    _vector_check(A, Bt, C2, True, 2048, seed=3, scale=3.0)

    Ai, Bti = workload_refs.operands("transb2048", "ints")
    refi = workload_refs.reference("transb2048", "ints")
    dAi, dBti = dev(Ai), dev(Bti)
    dC.fill_(float("nan"))
    binding.gemm_f32(dAi, dBti, dC, transB=True)
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), refi)
    binding.pack_b(dBti, dBp, transB=True)
    dC2.fill_(float("nan"))
    binding.gemm_f32_packed(dAi, dBp, dC2)
    assert np.array_equal(dC2.cpu().numpy().astype(np.float64), refi)


@pytest.mark.parametrize("N,K,transB,pad", [(130, 70, False, 0), (130, 70, True, 3), (64, 9, False, 5),
                                            (300, 257, True, 0), (1, 1, False, 0)])
def test_pack_b_bit_exact_and_packed_product(N, K, transB, pad):
    P = binding.pack_b_panel_width()
    B = synth.uniform((N, K) if transB else (K, N), 70, synth.TENSOR_B)
    dB, _ = padded_dev(B, pad)
    dBp = torch.full((binding.pack_b_size(N, K) // 4,), float("nan"), device="cuda")
    binding.pack_b(dB, dBp, transB=transB)
    want = oracle.pack_b(B, P, transB=transB)
    got = dBp.cpu().numpy().reshape(want.shape)
    assert np.array_equal(got, want) and not np.signbit(got[:, :, :][got == 0]).any()
    for M in (1, 67, 200):
        A = synth.uniform((M, K), 71, synth.TENSOR_A)
        for apad in (0, 3):
            dA, _ = padded_dev(A, apad)
            dC, bufC = padded_dev(np.full((M, N), np.nan, np.float32), apad)
            binding.gemm_f32_packed(dA, dBp, dC)
            whole = bufC.cpu().numpy()
            check_close(whole[:, :N], oracle.gemm_f32_packed(A, want, N), K)
            assert np.isnan(whole[:, N:]).all()
    Ai = synth.small_ints((90, K), 72, synth.TENSOR_A)
    Bi = synth.small_ints((N, K) if transB else (K, N), 72, synth.TENSOR_B)
    binding.pack_b(dev(Bi), dBp, transB=transB)
    dC = torch.empty((90, N), device="cuda")
    binding.gemm_f32_packed(dev(Ai), dBp, dC)
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), oracle.gemm_f32(Ai, Bi, transB=transB))


def test_workload_batched64_full_oracle():
    A, B = synth.make_operands("batched64")
    ref = oracle.gemm_f32_batched(A, B, nthreads=NTHREADS)
    dC = torch.full((4096, 64, 64), float("nan"), device="cuda")
    binding.gemm_f32_batched(dev(A), dev(B), dC)
    C = dC.cpu().numpy()
    assert np.isfinite(C).all()
    diff = np.abs(C.astype(np.float64) - ref)
    assert diff.max() <= 1e-3 * math.sqrt(64 / 1024.0)
    per_batch = np.sqrt((diff ** 2).sum(axis=(1, 2))) / np.sqrt((ref ** 2).sum(axis=(1, 2)))
    assert per_batch.max() <= 1e-5


def test_batched_integer_bit_exact_ragged_and_transb():
    for transB in (False, True):
        A = synth.small_ints((37, 50, 70), 80, synth.TENSOR_A)
        B = synth.small_ints((37, 45, 70) if transB else (37, 70, 45), 80, synth.TENSOR_B)
        ref = oracle.gemm_f32_batched(A, B, transB=transB, nthreads=NTHREADS)
        dC = torch.full((37, 50, 45), float("nan"), device="cuda")
        binding.gemm_f32_batched(dev(A), dev(B), dC, transB=transB)
        assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)


def test_batched_poisoned_neighbour_does_not_leak():
    A = synth.uniform((9, 64, 64), 81, synth.TENSOR_A)
    B = synth.uniform((9, 64, 64), 81, synth.TENSOR_B)
    ref = oracle.gemm_f32_batched(A, B)
    A[4] = np.nan
    dC = torch.empty((9, 64, 64), device="cuda")
    binding.gemm_f32_batched(dev(A), dev(B), dC)
    C = dC.cpu().numpy()
    assert np.isnan(C[4]).all()
    for b in (3, 5):
        check_close(C[b], ref[b], 64)


@pytest.mark.parametrize("transB", [False, True])
def test_batched64_streaming_path_many_products_bit_exact(transB):
    """More products than resident workgroups (each workgroup walks several), a count that is
    not a multiple of the grid, padded leading dimensions and batch strides, NaN in all padding."""
    batch = 1100
    A = synth.small_ints((batch, 64, 64), 82, synth.TENSOR_A)
    B = synth.small_ints((batch, 64, 64), 82, synth.TENSOR_B)
    ref = oracle.gemm_f32_batched(A, B, transB=transB, nthreads=NTHREADS)
    bufA = torch.full((batch, 66, 68), float("nan"), device="cuda")
    bufB = torch.full((batch, 65, 72), float("nan"), device="cuda")
    bufC = torch.full((batch, 67, 68), float("nan"), device="cuda")
    dA, dB, dC = bufA[:, :64, :64], bufB[:, :64, :64], bufC[:, :64, :64]
    dA.copy_(torch.from_numpy(A))
    dB.copy_(torch.from_numpy(B))
    binding.gemm_f32_batched(dA, dB, dC, transB=transB)
    whole = bufC.cpu().numpy()
    assert np.array_equal(whole[:, :64, :64].astype(np.float64), ref)
    assert np.isnan(whole[:, 64:, :]).all() and np.isnan(whole[:, :, 64:]).all()
    # the same products through the general tiled kernel agree bit for bit in the exact regime
    binding.set_test_hooks(force_tile=3)
    try:
        dC2 = torch.full((batch, 64, 64), float("nan"), device="cuda")
        binding.gemm_f32_batched(dA, dB, dC2, transB=transB)
        assert np.array_equal(dC2.cpu().numpy().astype(np.float64), ref)
    finally:
        binding.set_test_hooks(force_tile=None)


def test_batched64_uniform_values_and_two_products():
    for batch in (2, 3, 513):
        A = synth.uniform((batch, 64, 64), 83, synth.TENSOR_A)
        B = synth.uniform((batch, 64, 64), 83, synth.TENSOR_B)
        ref = oracle.gemm_f32_batched(A, B, nthreads=NTHREADS)
        dC = torch.full((batch, 64, 64), float("nan"), device="cuda")
        binding.gemm_f32_batched(dev(A), dev(B), dC)
        C = dC.cpu().numpy()
        for b in range(batch):
            check_close(C[b], ref[b], 64)


# --------------------------------------------------------------------- split-K (few tiles, long K)

@pytest.mark.parametrize("transB", [False, True])
def test_split_k_small_outputs_long_k(transB):
    """Outputs too small to occupy the chip: the dispatcher splits K; the second pass sums the
    partial products in a fixed order.  Ragged M, N and K, padded C with NaN guards."""
    for idx, (M, N, K) in enumerate([(128, 128, 8192), (100, 70, 5003), (64, 64, 4096), (33, 257, 3000),
                                      (1, 1, 1000003), (3, 5, 300001), (40, 2, 150000)]):
        name = binding.variant_name(M, N, K, transB=transB)
        assert "splitk" in name, name
        print(f"split-K {name} M={M} N={N} K={K} transB={transB}", flush=True)
        A = synth.uniform((M, K), 700 + idx, synth.TENSOR_A)
        B = synth.uniform((N, K) if transB else (K, N), 700 + idx, synth.TENSOR_B)
        ref = oracle.gemm_f32(A, B, transB=transB, nthreads=NTHREADS)
        dC, bufC = padded_dev(np.full((M, N), np.nan, np.float32), 3)
        binding.gemm_f32(dev(A), dev(B), dC, transB=transB)
        whole = bufC.cpu().numpy()
        check_close(whole[:, :N], ref, K)
        assert np.isnan(whole[:, N:]).all()


@pytest.mark.parametrize("split", [2, 3, 5, 16])
def test_split_k_forced_factors_bit_exact_and_deterministic(split):
    """Any split factor gives the exact result on integer operands (also through packed B), and the
    same bits on every run for float operands."""
    binding.set_test_hooks(force_split=split)
    try:
        M, N, K = 150, 200, 2000
        A = synth.small_ints((M, K), 710, synth.TENSOR_A)
        B = synth.small_ints((K, N), 710, synth.TENSOR_B)
        ref = oracle.gemm_f32(A, B, nthreads=NTHREADS)
        dA, dB = dev(A), dev(B)
        dC = torch.full((M, N), float("nan"), device="cuda")
        binding.gemm_f32(dA, dB, dC)
        assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)
        dC.fill_(float("nan"))
        binding.gemm_f32(dA, dev(B.T), dC, transB=True)
        assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)
        dBp = torch.empty(binding.pack_b_size(N, K) // 4, device="cuda")
        binding.pack_b(dB, dBp)
        dC.fill_(float("nan"))
        binding.gemm_f32_packed(dA, dBp, dC)
        assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)
        Af = synth.uniform((M, K), 711, synth.TENSOR_A)
        Bf = synth.uniform((K, N), 711, synth.TENSOR_B)
        dAf, dBf = dev(Af), dev(Bf)
        outs = []
        for _ in range(3):
            dC.fill_(float("nan"))
            binding.gemm_f32(dAf, dBf, dC)
            outs.append(dC.cpu().numpy())
        assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
        check_close(outs[0], oracle.gemm_f32(Af, Bf, nthreads=NTHREADS), K)
    finally:
        binding.set_test_hooks(force_split=None)


def test_shutdown_releases_workspace_and_library_stays_usable():
    A = synth.uniform((64, 4096), 720, synth.TENSOR_A)
    B = synth.uniform((4096, 64), 720, synth.TENSOR_B)
    ref = oracle.gemm_f32(A, B, nthreads=NTHREADS)
    dC = torch.empty((64, 64), device="cuda")
    for _ in range(2):
        binding.gemm_f32(dev(A), dev(B), dC)
        check_close(dC.cpu().numpy(), ref, 4096)
        torch.cuda.synchronize()
        binding.lib().gemm_f32_shutdown()

# --------------------------------------------------------------------- split tail (uneven tile counts)

@pytest.mark.parametrize("tile,how", [("t128", "tail"), ("t64", "tail"), ("tb64", "tail"), ("t64", "quad"), ("tb64", "quad"),
                                      ("t128x64", "quad"), ("t64x128", "quad"), ("tq32", "tail"), ("tq64x32", "tail"), ("tq32x64", "tail")])
@pytest.mark.parametrize("transB", [False, True])
def test_split_tail_bit_exact(force_tile, tile, how, transB):
    """More tiles than one round of 256, with a small remainder.  "tail": the remainder's tiles are cut
    along K and summed by a second pass.  "quad": they are cut into 32 x 32 blocks, each computed by a
    whole workgroup whose waves share the slabs along k and add up through LDS.  Exact on integer
    operands; ragged edges (blocks of edge tiles that lie outside the matrix), a K tail, padded C."""
    force_tile(tile)
    binding.set_test_hooks(no_strip=True)          # these shapes would hand their last columns to the strip
    if how == "tail":
        binding.set_test_hooks(no_quad=True)
    shapes = {"t128": [(2100, 2200, 1000)], "t64": [(1000, 1030, 999), (1030, 1100, 1100)],
              "tb64": [(1000, 1030, 999), (1030, 1100, 1100)], "t128x64": [(2000, 1090, 1100), (2200, 1000, 333)],
              "t64x128": [(1090, 2000, 1100)], "tq32": [(520, 530, 3000), (576, 570, 4100)], "tq64x32": [(770, 760, 2100), (1030, 520, 3000)],
              "tq32x64": [(770, 760, 2100), (1030, 520, 3000)]}[tile]
    try:
        _split_tail_cases(shapes, how, transB)
    finally:
        binding.set_test_hooks()


def _split_tail_cases(shapes, how, transB):
    for idx, (M, N, K) in enumerate(shapes):
        name = binding.variant_name(M, N, K, transB=transB)
        assert "/" + how in name, name
        print(f"split tail {name} M={M} N={N} K={K}", flush=True)
        A = synth.small_ints((M, K), 800 + idx, synth.TENSOR_A)
        B = synth.small_ints((N, K) if transB else (K, N), 800 + idx, synth.TENSOR_B)
        ref = oracle.gemm_f32(A, B, transB=transB, nthreads=NTHREADS)
        dC, bufC = padded_dev(np.full((M, N), np.nan, np.float32), 2)
        binding.gemm_f32(dev(A), dev(B), dC, transB=transB)
        whole = bufC.cpu().numpy()
        assert np.array_equal(whole[:, :N].astype(np.float64), ref)
        assert np.isnan(whole[:, N:]).all()


def test_split_tail_ragged_workload_parity_determinism_and_packed():
    """The ragged workload (272 tiles of 64x64) takes this path: 32 x 32 blocks by default, K ranges
    when those are switched off, whole tiles when both are."""
    binding.set_test_hooks(no_strip=True)          # (by default the six columns behind 16 tile columns are a strip)
    assert "/quad16" in binding.variant_name(1000, 1030, 999)
    A, B = synth.make_operands("ragged")
    ref = oracle.gemm_f32(A, B, nthreads=NTHREADS)
    dA, dB = dev(A), dev(B)
    outs = []
    for _ in range(3):
        dC = torch.full((1000, 1030), float("nan"), device="cuda")
        binding.gemm_f32(dA, dB, dC)
        outs.append(dC.cpu().numpy())
    check_close(outs[0], ref, 999)
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    dBp = torch.empty(binding.pack_b_size(1030, 999) // 4, device="cuda")
    binding.pack_b(dB, dBp)
    dC = torch.full((1000, 1030), float("nan"), device="cuda")
    binding.gemm_f32_packed(dA, dBp, dC)
    check_close(dC.cpu().numpy(), ref, 999)
    binding.set_test_hooks(no_quad=True)
    binding.set_test_hooks(no_kshare=True)  # or the tile whose waves share the slabs takes the shape whole
    try:
        assert "/tail16x8" in binding.variant_name(1000, 1030, 999)
        dC.fill_(float("nan"))
        binding.gemm_f32(dA, dB, dC)
        check_close(dC.cpu().numpy(), ref, 999)
    finally:
        binding.set_test_hooks(no_quad=None)
        binding.set_test_hooks(no_kshare=None)
    binding.set_test_hooks(no_tail_split=True)
    try:
        name = binding.variant_name(1000, 1030, 999)
        assert "/tail" not in name and "/quad" not in name
        dC.fill_(float("nan"))
        binding.gemm_f32(dA, dB, dC)
        check_close(dC.cpu().numpy(), ref, 999)
    finally:
        binding.set_test_hooks()


STRIP_TILES = ["t64", "tb64", "t128", "t128x64", "t64x128", "t128x32", "t32x128", "t256", "t256x128", "t128x256"]


@pytest.mark.parametrize("tile", STRIP_TILES)
@pytest.mark.parametrize("transB", [False, True])
def test_strip_columns_bit_exact(force_tile, tile, transB):
    """N a few columns (1..8) more than whole tiles: the tiles stop at the last tile boundary and the columns
    behind it are computed in the vector unit by extra workgroups of the same launch.  Row counts that are not
    multiples of the 16 rows a strip workgroup takes, K below one request, ragged, and longer than what the strip
    stages in LDS at a time; integer operands (exact), NaN in old C and in the padding of all three matrices."""
    force_tile(tile)
    # (a long K with a small output would otherwise be split into ranges; and where the edge tile column fits the
    # round the cost model would keep it)
    binding.set_test_hooks(force_split=1, force_strip=True)
    BM, BN = TILE_DIMS[tile]
    cases = [(BM * 2 + 5, BN + 1, 77), (37, BN + 3, 300), (16, 2 * BN + 4, 1), (130, BN + 5, 2500), (BM + 17, BN + 8, 1031),
             (70, BN + 3, 0)]
    for idx, (M, N, K) in enumerate(cases):
        name = binding.variant_name(M, N, K, transB=transB)
        print(f"strip case tile={tile} transB={transB} M={M} N={N} K={K} {name}", flush=True)
        assert f"/strip{N % BN}" in name, name
        A = synth.small_ints((M, K), 600 + idx, synth.TENSOR_A)
        B = synth.small_ints((N, K) if transB else (K, N), 600 + idx, synth.TENSOR_B)
        ref = oracle.gemm_f32(A, B, transB=transB, nthreads=NTHREADS)
        dA, _ = padded_dev(A, 3)
        dB, _ = padded_dev(B, 5)
        dC, bufC = padded_dev(np.full((M, N), np.nan, np.float32), 2)
        binding.gemm_f32(dA, dB, dC, transB=transB)
        whole = bufC.cpu().numpy()
        assert np.array_equal(whole[:, :N].astype(np.float64), ref)
        assert np.isnan(whole[:, N:]).all(), "ldc padding was written"
    binding.set_test_hooks()


@pytest.mark.parametrize("transB", [False, True])
@pytest.mark.parametrize("rows", [1, 2, 4])
def test_strip_rows_per_wave_and_pause(rows, transB):
    """The strip with one, two and four rows of C per wave (the library picks by M), with and without the pause
    before its first load, narrow (S <= 4) and wide: integer operands, exact; row counts that leave the last
    workgroup partly empty; K of several chunks with a ragged end."""
    try:
        for wait in (0, 3):
            binding.set_test_hooks(force_tile=3, force_strip=True, force_split=1, strip_rows=rows, strip_wait=wait)  # the 64x64x64 tile
            for idx, (M, N, K) in enumerate([(4 * rows * 5 + 3, 64 + 3, 2100), (97, 128 + 7, 1025), (8, 64 + 8, 513)]):
                name = binding.variant_name(M, N, K, transB=transB)
                print(f"strip rows={rows} wait={wait} transB={transB} M={M} N={N} K={K} {name}", flush=True)
                assert "/strip" in name, name
                A = synth.small_ints((M, K), 650 + idx, synth.TENSOR_A)
                B = synth.small_ints((N, K) if transB else (K, N), 650 + idx, synth.TENSOR_B)
                ref = oracle.gemm_f32(A, B, transB=transB, nthreads=NTHREADS)
                dA, _ = padded_dev(A, 3)
                dB, _ = padded_dev(B, 5)
                dC, bufC = padded_dev(np.full((M, N), np.nan, np.float32), 2)
                binding.gemm_f32(dA, dB, dC, transB=transB)
                whole = bufC.cpu().numpy()
                assert np.array_equal(whole[:, :N].astype(np.float64), ref)
                assert np.isnan(whole[:, N:]).all(), "ldc padding was written"
    finally:
        binding.set_test_hooks()


@pytest.mark.parametrize("tile,split", [("t128x256", 3), ("t128x256", 6), ("t256", 3), ("t256x128", 3)])
def test_wide_tiles_two_to_a_compute_unit_stores_exact(tile, split):
    """Tiles 256 columns wide store 16 bytes per lane and row.  With more workgroups than compute units, two of
    them share one and their epilogues run against each other's loads: the stores then have to be complete before
    their data registers are written again (the 128 x 256 tile once stored the next row's value in the fourth dword
    of some lanes, differently from run to run).  Integer operands, K split so that every tile goes through the
    workspace, N not a multiple of the tile: exact, on three launches in a row."""
    M, N, K = 2798, 1582, 889
    try:
        binding.set_test_hooks(force_tile=TILES[tile], force_split=split)
        name = binding.variant_name(M, N, K)
        print(f"{tile} split={split} {name}", flush=True)
        assert f"splitk{split}" in name, name
        A = synth.small_ints((M, K), 760, synth.TENSOR_A)
        B = synth.small_ints((K, N), 760, synth.TENSOR_B)
        ref = oracle.gemm_f32(A, B, nthreads=NTHREADS)
        dA, dB = dev(A), dev(B)
        for launch in range(3):
            dC = torch.full((M, N), float("nan"), device="cuda")
            binding.gemm_f32(dA, dB, dC)
            assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref), f"launch {launch}"
    finally:
        binding.set_test_hooks()


def test_strip_uniform_operands_scalings_and_switch():
    """The ragged workload's own shape takes the strip (6 columns behind 16 whole tile columns): within
    tolerance on U(-1,1) operands, the same bits on every launch, alpha and beta applied, and the same product
    with the strip switched off (an edge tile column instead) agrees within tolerance."""
    M, N, K = 1000, 1030, 999
    assert binding.variant_name(M, N, K).endswith("/strip6")
    A, B = synth.make_operands("ragged")
    ref = oracle.gemm_f32(A, B, nthreads=NTHREADS)
    dA, dB = dev(A), dev(B)
    outs = []
    for _ in range(3):
        dC = torch.full((M, N), float("nan"), device="cuda")
        binding.gemm_f32(dA, dB, dC)
        outs.append(dC.cpu().numpy())
    check_close(outs[0], ref, K)
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    C0 = synth.uniform((M, N), 77, synth.TENSOR_X)
    dC = dev(C0)
    binding.gemm_f32_ex(dA, dB, dC, alpha=-2.0, beta=0.5)
    want = -2.0 * ref + 0.5 * C0.astype(np.float64)
    assert np.abs(dC.cpu().numpy().astype(np.float64) - want).max() <= 2.5e-3
    binding.set_test_hooks(no_strip=True)
    try:
        assert "/strip" not in binding.variant_name(M, N, K)
        dC = torch.full((M, N), float("nan"), device="cuda")
        binding.gemm_f32(dA, dB, dC)
        check_close(dC.cpu().numpy(), ref, K)
    finally:
        binding.set_test_hooks(no_strip=None)


def test_mfma_rate_probe_runs_and_validates_its_arguments():
    lib = binding.lib()
    ops = torch.zeros(512, device="cuda")
    sink = torch.full((4,), 7.0, device="cuda")
    binding.gemm_f32_mfma_rate_probe(1024, ops, sink)
    torch.cuda.synchronize()
    assert torch.equal(sink, torch.full((4,), 7.0, device="cuda"))       # the sink is never written
    assert lib.gemm_f32_mfma_rate_probe(1000, ops.data_ptr(), sink.data_ptr()) == -1    # not a multiple of 16
    assert lib.gemm_f32_mfma_rate_probe(0, ops.data_ptr(), sink.data_ptr()) == -1
    assert lib.gemm_f32_mfma_rate_probe(1024, None, sink.data_ptr()) == -2
    assert lib.gemm_f32_mfma_rate_probe(1024, ops.data_ptr(), None) == -2
