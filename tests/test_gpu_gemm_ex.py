"""GPU parity of the general form  C = alpha*op(A)*op(B) + beta*C  (gemm_f32_ex, gemm_f32_ex_batched,
through the C ABI) against the general-form CPU oracle on the same seeded inputs.

Tolerance.  The product part carries the plain product's bound scaled by |alpha|
(|alpha| * 1e-3 * sqrt(K/1024) for U(-1,1) operands); the epilogue adds two fp32 multiplications
and one addition (or one fused multiply-add), each rounding relative 2^-24 of values bounded by
|alpha|*|sum| + |beta|*|C_old|, i.e. at most 3 * 2^-24 * (|alpha|*K + |beta|*max|C_old|) -- far
below the first term for the sizes here; the tests allow the sum of both.  Integer-valued operands
with integer alpha, beta are exact and compared bit for bit."""
from __future__ import annotations

import math
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_2002_02268_amd import binding, synth  # noqa: E402

from test_gpu_parity import NTHREADS, TILES, TILE_DIMS, dev, padded_dev  # noqa: E402

FLAGS = [(False, False), (False, True), (True, False), (True, True)]
TENSOR_C = 2


def stored(X, trans):
    return np.ascontiguousarray(X.T) if trans else X


def tolerance(K, alpha, beta, c_max):
    return abs(alpha) * 1e-3 * math.sqrt(max(K, 1) / 1024.0) + 3 * 2.0 ** -24 * (abs(alpha) * K + abs(beta) * c_max)


@pytest.fixture
def force_tile():
    def _set(name):
        binding.set_test_hooks(force_tile=TILES[name])
    yield _set
    binding.set_test_hooks(force_tile=None)


SHAPES = [(1, 1, 1), (33, 65, 17), (130, 257, 70), (300, 513, 129), (257, 130, 1), (5, 700, 33), (700, 5, 40)]


@pytest.mark.parametrize("tile", list(TILES))
@pytest.mark.parametrize("tA,tB", FLAGS)
def test_ex_small_shapes_every_tile(force_tile, tile, tA, tB):
    """Ragged shapes, all four transpose combinations, padded rows everywhere (NaN in the padding),
    alpha and beta both non-trivial: within tolerance, and the ld padding of C survives."""
    force_tile(tile)
    alpha, beta = 1.25, -0.5
    for idx, (M, N, K) in enumerate(SHAPES):
        print(f"case tile={tile} tA={tA} tB={tB} M={M} N={N} K={K}", flush=True)
        A = synth.uniform((M, K), 800 + idx, synth.TENSOR_A)
        B = synth.uniform((K, N), 800 + idx, synth.TENSOR_B)
        C0 = synth.uniform((M, N), 800 + idx, TENSOR_C)
        ref = oracle.gemm_f32_ex(stored(A, tA), stored(B, tB), C0, alpha, beta, tA, tB, nthreads=NTHREADS)
        dA, _ = padded_dev(stored(A, tA), 3)
        dB, _ = padded_dev(stored(B, tB), 5)
        dC, bufC = padded_dev(C0, 2)
        binding.gemm_f32_ex(dA, dB, dC, alpha, beta, tA, tB)
        whole = bufC.cpu().numpy()
        err = np.abs(whole[:, :N].astype(np.float64) - ref).max(initial=0.0)
        assert err <= tolerance(K, alpha, beta, 1.0), err
        assert np.isnan(whole[:, N:]).all(), "ldc padding was written"


@pytest.mark.parametrize("tile", list(TILES))
@pytest.mark.parametrize("tB", [False, True])
def test_ex_transposed_a_boundary_sweep_bit_exact(force_tile, tile, tB):
    """A stored K x M with M and N around tile multiples: edge tiles shorter than a tile (clamped
    element loads along the contiguous dimension of A) and edge tiles moved back inside.  Integer
    operands, integer alpha and beta: exact."""
    force_tile(tile)
    BM, BN = TILE_DIMS[tile]
    K = 37
    for M in (BM - 1, BM, BM + 1, 2 * BM + 7):
        for N in (BN - 3, BN + 2):
            print(f"case tile={tile} tB={tB} M={M} N={N}", flush=True)
            A = synth.small_ints((M, K), 820 + M, synth.TENSOR_A)
            B = synth.small_ints((K, N), 820 + N, synth.TENSOR_B)
            C0 = synth.small_ints((M, N), 820, TENSOR_C, -9, 9)
            ref = oracle.gemm_f32_ex(stored(A, True), stored(B, tB), C0, 2.0, -3.0, True, tB, nthreads=NTHREADS)
            dA, _ = padded_dev(stored(A, True), 1)
            dC, bufC = padded_dev(C0, 3)
            binding.gemm_f32_ex(dA, dev(stored(B, tB)), dC, 2.0, -3.0, True, tB)
            whole = bufC.cpu().numpy()
            assert np.array_equal(whole[:, :N].astype(np.float64), ref)
            assert np.isnan(whole[:, N:]).all()


def test_ex_default_scalars_equal_plain_entry_point_bit_for_bit():
    for tB in (False, True):
        M, N, K = 300, 260, 150
        A = synth.uniform((M, K), 840, synth.TENSOR_A)
        B = synth.uniform((K, N), 840, synth.TENSOR_B)
        dA, dB = dev(A), dev(stored(B, tB))
        C1 = torch.full((M, N), float("nan"), device="cuda")
        C2 = torch.full((M, N), float("nan"), device="cuda")
        binding.gemm_f32(dA, dB, C1, transB=tB)
        binding.gemm_f32_ex(dA, dB, C2, 1.0, 0.0, False, tB)
        assert torch.equal(C1, C2)
        # A stored K x M holds the same values: same k order per element, same bits
        C3 = torch.full((M, N), float("nan"), device="cuda")
        binding.gemm_f32_ex(dev(stored(A, True)), dB, C3, 1.0, 0.0, True, tB)
        assert torch.equal(C1, C3)


def test_ex_beta_zero_never_reads_c_and_alpha_zero_keeps_beta_c():
    M, N, K = 200, 180, 64
    A = synth.uniform((M, K), 850, synth.TENSOR_A)
    B = synth.uniform((K, N), 850, synth.TENSOR_B)
    C0 = synth.uniform((M, N), 850, TENSOR_C)
    dC = torch.full((M, N), float("nan"), device="cuda")
    binding.gemm_f32_ex(dev(A), dev(B), dC, 0.75, 0.0)
    got = dC.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert np.abs(got - oracle.gemm_f32_ex(A, B, None, 0.75, 0.0)).max() <= tolerance(K, 0.75, 0, 0)
    dC = dev(C0)
    binding.gemm_f32_ex(dev(A), dev(B), dC, 0.0, 2.0)          # power of two: exact
    assert np.array_equal(dC.cpu().numpy(), 2.0 * C0)
    # K == 0: C = beta * C
    dC = dev(C0)
    binding.gemm_f32_ex(torch.empty((M, 0), device="cuda"), torch.empty((0, N), device="cuda"), dC, 3.0, 0.5)
    assert np.array_equal(dC.cpu().numpy(), 0.5 * C0)
    dC = torch.full((M, N), float("nan"), device="cuda")
    binding.gemm_f32_ex(torch.empty((M, 0), device="cuda"), torch.empty((0, N), device="cuda"), dC, 3.0, 0.0)
    assert np.array_equal(dC.cpu().numpy(), np.zeros((M, N), np.float32))


@pytest.mark.parametrize("tA,tB", FLAGS)
def test_ex_split_k_and_split_last_round_apply_scalars_once(tA, tB):
    """Shapes that take the K-split path (small output, long K) and the split last round
    (272 tiles): the second pass applies alpha and beta; integer operands, exact."""
    for (M, N, K) in [(96, 80, 4000), (1000, 1030, 999)]:
        A = synth.small_ints((M, K), 860, synth.TENSOR_A)
        B = synth.small_ints((K, N), 860, synth.TENSOR_B)
        C0 = synth.small_ints((M, N), 860, TENSOR_C, -9, 9)
        ref = oracle.gemm_f32_ex(stored(A, tA), stored(B, tB), C0, -2.0, 3.0, tA, tB, nthreads=NTHREADS)
        for no_quad in (False, True):       # the last round as 32 x 32 blocks (scalars applied in the kernel), then as K ranges
            if no_quad:
                binding.set_test_hooks(no_quad=True)
                binding.set_test_hooks(no_kshare=True)  # or the shared-slab tile would take the ragged shape whole
            binding.set_test_hooks(no_strip=True)       # the last columns as an edge tile column: this test is about the split round
            try:
                name = binding.variant_name(M, N, K, transB=tB)
                print(f"case tA={tA} tB={tB} M={M} N={N} K={K} variant={name}", flush=True)
                assert ("splitk" in name) or ("tail" in name) or ("quad" in name and not no_quad)
                dC = dev(C0)
                binding.gemm_f32_ex(dev(stored(A, tA)), dev(stored(B, tB)), dC, -2.0, 3.0, tA, tB)
            finally:
                binding.set_test_hooks()
            assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)


def test_ex_ragged_workload_transposed_a_within_tolerance():
    w = synth.WORKLOADS["ragged"]
    M, N, K = w["M"], w["N"], w["K"]
    A = synth.uniform((M, K), 870, synth.TENSOR_A)
    B = synth.uniform((K, N), 870, synth.TENSOR_B)
    C0 = synth.uniform((M, N), 870, TENSOR_C)
    ref = oracle.gemm_f32_ex(stored(A, True), B, C0, 1.5, 0.25, True, False, nthreads=NTHREADS)
    dC = dev(C0)
    binding.gemm_f32_ex(dev(stored(A, True)), dev(B), dC, 1.5, 0.25, True, False)
    got = dC.cpu().numpy().astype(np.float64)
    assert np.abs(got - ref).max() <= tolerance(K, 1.5, 0.25, 1.0)
    assert np.linalg.norm(got - ref) / np.linalg.norm(ref) <= 1e-5


@pytest.mark.parametrize("tA,tB", FLAGS)
def test_ex_batched_non_contiguous_strides(tA, tB):
    """Batches taken as every second product of a larger buffer with padded rows (batch stride
    larger than one product, leading dimensions larger than the rows); the skipped products hold
    NaN (inputs) or a sentinel (outputs) that must survive."""
    batch, M, N, K = 5, 70, 90, 50
    alpha, beta = 2.0, -1.0
    A = synth.small_ints((batch, M, K), 880, synth.TENSOR_A)
    B = synth.small_ints((batch, K, N), 880, synth.TENSOR_B)
    C0 = synth.small_ints((batch, M, N), 880, TENSOR_C, -9, 9)
    As = np.ascontiguousarray(A.transpose(0, 2, 1)) if tA else A
    Bs = np.ascontiguousarray(B.transpose(0, 2, 1)) if tB else B

    def spaced(x, fill):
        buf = torch.full((2 * x.shape[0], x.shape[1], x.shape[2] + 3), fill, dtype=torch.float32, device="cuda")
        view = buf[::2, :, : x.shape[2]]
        view.copy_(torch.from_numpy(x))
        return view, buf

    dA, _ = spaced(As, float("nan"))
    dB, _ = spaced(Bs, float("nan"))
    dC, bufC = spaced(C0, 777.0)
    binding.gemm_f32_ex_batched(dA, dB, dC, alpha, beta, tA, tB)
    whole = bufC.cpu().numpy()
    for b in range(batch):
        ref = oracle.gemm_f32_ex(As[b], Bs[b], C0[b], alpha, beta, tA, tB)
        assert np.array_equal(whole[2 * b, :, :N].astype(np.float64), ref), b
    assert (whole[1::2] == 777.0).all() and (whole[:, :, N:] == 777.0).all()


def test_ex_batched_default_scalars_take_the_streaming_path_and_match():
    batch = 64
    A = synth.uniform((batch, 64, 64), 890, synth.TENSOR_A)
    B = synth.uniform((batch, 64, 64), 890, synth.TENSOR_B)
    C1 = torch.empty((batch, 64, 64), device="cuda")
    C2 = torch.empty((batch, 64, 64), device="cuda")
    binding.gemm_f32_batched(dev(A), dev(B), C1)
    binding.gemm_f32_ex_batched(dev(A), dev(B), C2)
    assert torch.equal(C1, C2)
    C3 = dev(np.ones((batch, 64, 64), np.float32))
    binding.gemm_f32_ex_batched(dev(A), dev(B), C3, 1.0, 1.0)
    ref = oracle.gemm_f32_batched(A, B, nthreads=NTHREADS) + 1.0
    assert np.abs(C3.cpu().numpy().astype(np.float64) - ref).max() <= tolerance(64, 1.0, 1.0, 1.0)


def test_ex_error_codes():
    lib = binding.lib()
    a = torch.zeros(4096, device="cuda")
    b = torch.zeros(4096, device="cuda")
    c = torch.zeros(4096, device="cuda")
    ap, bp, cp = a.data_ptr(), b.data_ptr(), c.data_ptr()
    ok = lambda *args: lib.gemm_f32_ex(*args)
    assert ok(8, 16, 4, 1.0, ap, 4, 0, bp, 16, 0, 0.0, cp, 16) == 0
    assert ok(8, 16, 4, 1.0, ap, 8, 1, bp, 16, 0, 0.0, cp, 16) == 0
    assert ok(8, 16, 4, 1.0, ap, 7, 1, bp, 16, 0, 0.0, cp, 16) == -1      # A stored K x M needs lda >= M
    assert ok(8, 16, 4, 1.0, ap, 3, 0, bp, 16, 0, 0.0, cp, 16) == -1
    assert ok(8, 16, 4, 1.0, ap, 4, 2, bp, 16, 0, 0.0, cp, 16) == -1      # flags are 0 or 1
    assert ok(8, 16, 4, 1.0, ap, 4, 0, bp, 16, 3, 0.0, cp, 16) == -1
    assert ok(8, 16, 4, 1.0, None, 4, 0, bp, 16, 0, 0.0, cp, 16) == -2
    assert ok(8, 16, 4, 1.0, ap, 4, 0, bp, 16, 0, 1.0, ap, 16) == -3
    assert ok(0, 16, 4, 1.0, None, 4, 0, None, 16, 0, 1.0, None, 16) == 0
    torch.cuda.synchronize()


def test_ex_many_seeded_shapes_bit_exact():
    """120 products whose shapes, strides, transpose flags and integer scalars are drawn from the
    counter-based generator (so the list is the same on every run): the dispatch picks tile, K split
    and split last round by itself; integer operands make every result exact."""
    draws = synth.small_ints((120, 12), 4242, 7, 0, 1 << 20).astype(np.int64)
    for case, d in enumerate(draws):
        d = [int(x) for x in d]
        M = 1 + d[0] % 700
        N = 1 + d[1] % 700
        K = 1 + (d[2] % 400 if d[3] % 4 else d[2] % 6000)        # every fourth case: long K
        if d[3] % 16 == 0:
            M, N = 1 + d[0] % 90, 1 + d[1] % 90                   # small outputs: K split
        tA, tB = bool(d[4] & 1), bool(d[4] & 2)
        alpha, beta = float(d[5] % 5 - 2), float(d[6] % 4 - 1)
        pads = (d[7] % 5, d[8] % 5, d[9] % 5)
        print(f"case {case}: M={M} N={N} K={K} tA={tA} tB={tB} alpha={alpha} beta={beta} pads={pads} "
              f"variant={binding.variant_name(M, N, K, transB=tB)}", flush=True)
        A = synth.small_ints((M, K), 3000 + case, synth.TENSOR_A)
        B = synth.small_ints((K, N), 3000 + case, synth.TENSOR_B)
        C0 = synth.small_ints((M, N), 3000 + case, TENSOR_C, -9, 9)
        ref = oracle.gemm_f32_ex(stored(A, tA), stored(B, tB), C0, alpha, beta, tA, tB, nthreads=NTHREADS)
        dA, _ = padded_dev(stored(A, tA), pads[0])
        dB, _ = padded_dev(stored(B, tB), pads[1])
        dC, bufC = padded_dev(C0, pads[2])
        binding.gemm_f32_ex(dA, dB, dC, alpha, beta, tA, tB)
        whole = bufC.cpu().numpy()
        assert np.array_equal(whole[:, :N].astype(np.float64), ref), case
        assert np.isnan(whole[:, N:]).all(), case


def test_ex_batched_many_seeded_shapes_bit_exact():
    """40 batched products with seeded shapes, batch counts, transpose flags, integer scalars, padded rows
    and batch strides larger than one product: exact on integer operands, padding and gaps untouched."""
    draws = synth.small_ints((40, 12), 5151, 7, 0, 1 << 20).astype(np.int64)
    for case, d in enumerate(draws):
        d = [int(x) for x in d]
        batch = 1 + d[0] % 9
        M, N, K = 1 + d[1] % 300, 1 + d[2] % 300, 1 + d[3] % 200
        if d[4] % 5 == 0:
            M = N = K = 64                                  # the streaming path when the scalars are (1, 0)
        tA, tB = bool(d[5] & 1), bool(d[5] & 2)
        alpha, beta = float(d[6] % 4 - 1), float(d[7] % 3 - 1)
        if d[4] % 10 == 0:
            tA, alpha, beta = False, 1.0, 0.0
        pad, gap = d[8] % 4, d[9] % 3
        print(f"case {case}: batch={batch} M={M} N={N} K={K} tA={tA} tB={tB} alpha={alpha} beta={beta} pad={pad} gap={gap}",
              flush=True)
        A = synth.small_ints((batch, M, K), 5200 + case, synth.TENSOR_A)
        B = synth.small_ints((batch, K, N), 5200 + case, synth.TENSOR_B)
        C0 = synth.small_ints((batch, M, N), 5200 + case, TENSOR_C, -9, 9)
        As = np.ascontiguousarray(A.transpose(0, 2, 1)) if tA else A
        Bs = np.ascontiguousarray(B.transpose(0, 2, 1)) if tB else B

        def spaced(x, fill):
            buf = torch.full(((1 + gap) * x.shape[0], x.shape[1], x.shape[2] + pad), fill, dtype=torch.float32,
                             device="cuda")
            view = buf[:: 1 + gap, :, : x.shape[2]]
            view.copy_(torch.from_numpy(x))
            return view, buf

        dA, _ = spaced(As, float("nan"))
        dB, _ = spaced(Bs, float("nan"))
        dC, bufC = spaced(C0, 555.0)
        binding.gemm_f32_ex_batched(dA, dB, dC, alpha, beta, tA, tB)
        whole = bufC.cpu().numpy()
        for b in range(batch):
            ref = oracle.gemm_f32_ex(As[b], Bs[b], C0[b], alpha, beta, tA, tB)
            assert np.array_equal(whole[(1 + gap) * b, :, :N].astype(np.float64), ref), (case, b)
        assert (whole[:, :, N:] == 555.0).all(), case
        if gap:
            keep = np.ones(whole.shape[0], bool)
            keep[:: 1 + gap] = False
            assert (whole[keep] == 555.0).all(), case



SKINNY = [
    # (M, N, K, transA, transB): at most 32 columns, or at most 32 rows, of C
    (700, 32, 2000, False, False), (700, 32, 2000, False, True), (1000, 17, 1537, False, False),
    (1000, 1, 4099, False, True), (257, 31, 513, False, False), (4096, 8, 600, False, True),
    (32, 900, 2000, False, True), (5, 1111, 3001, False, True), (32, 900, 2000, True, True),
    (1, 300, 5000, True, True), (16, 257, 512, False, True), (8, 4100, 1030, True, True),
    (2000, 24, 700, True, False), (3, 2000, 900, False, False),
]


@pytest.mark.parametrize("M,N,K,tA,tB", SKINNY)
def test_ex_products_with_one_short_dimension_match(M, N, K, tA, tB):
    """One dimension of C at most 32, through the dispatch's choice and through the tile that is 32
    wide in that dimension (four waves side by side along the other).  Rows and columns that do not fill the tile, K not a
    multiple of the slab, K split or not, padded strides, alpha and beta: exact on integers, within
    tolerance on U(-1,1)."""
    narrow_tiles = ("8" if N <= 32 else "9", "10")         # tile 128x32x32 / 32x128x32, and the 32x32 block with shared slabs
    for ints in (True, False):
        gen = synth.small_ints if ints else synth.uniform
        A = gen((M, K), 7000 + M, synth.TENSOR_A)
        B = gen((K, N), 7000 + N, synth.TENSOR_B)
        C0 = synth.small_ints((M, N), 7000, TENSOR_C, -9, 9)
        for alpha, beta in ((1.0, 0.0), (2.0, -1.0)):
            print(f"case M={M} N={N} K={K} tA={tA} tB={tB} ints={ints} alpha={alpha} beta={beta}", flush=True)
            ref = oracle.gemm_f32_ex(stored(A, tA), stored(B, tB), C0, alpha, beta, tA, tB, nthreads=NTHREADS)
            dA, _ = padded_dev(stored(A, tA), 3)
            dB, _ = padded_dev(stored(B, tB), 1)
            dC, bufC = padded_dev(C0 if beta else np.full((M, N), np.nan, np.float32), 2)
            for forced in (None,) + narrow_tiles:          # the dispatch's own choice, then the narrow tiles
                if forced is not None:
                    binding.set_test_hooks(force_tile=forced)
                    dC, bufC = padded_dev(C0 if beta else np.full((M, N), np.nan, np.float32), 2)
                try:
                    binding.gemm_f32_ex(dA, dB, dC, alpha, beta, tA, tB)
                finally:
                    binding.set_test_hooks(force_tile=None)
                whole = bufC.cpu().numpy()
                got = whole[:, :N].astype(np.float64)
                if ints:
                    assert np.array_equal(got, ref)
                else:
                    assert np.abs(got - ref).max() <= tolerance(K, alpha, beta, 9.0)
                assert np.isnan(whole[:, N:]).all(), "ldc padding was written"


def _strided_dev(X: np.ndarray, ld: int):
    """X (rows x cols) on the device inside a buffer whose rows are ld floats apart; the gaps hold NaN."""
    rows, cols = X.shape
    buf = torch.full(((rows - 1) * ld + cols,), float("nan"), device="cuda")
    view = torch.as_strided(buf, (rows, cols), (ld, 1))
    view.copy_(torch.from_numpy(X).cuda())
    return view, buf


@pytest.mark.parametrize("tile", ["t256", "t64", "t128x32"])
def test_leading_dimensions_beyond_32_bit_tile_offsets(force_tile, tile):
    """Leading dimensions so large that the byte offsets inside one tile exceed 32 bits: the kernels
    then take the per-lane 64-bit pointer path for every tile (interior, edge, ragged K).  A stored
    M x K with lda = 2^30 / (BM - 1) + 1000, B stored N x K with a matching ldb, then A stored K x M."""
    BM, BN = TILE_DIMS[tile]
    M, N, K = BM + 44, 150, 40
    wide_a = (1 << 30) // (BM - 1) + 1000
    wide_b = (1 << 30) // (BN - 1) + 1000
    A = synth.small_ints((M, K), 7300, synth.TENSOR_A)
    B = synth.small_ints((K, N), 7300, synth.TENSOR_B)
    ref = oracle.gemm_f32_ex(A, B, np.zeros((M, N), np.float32), 1.0, 0.0, False, False, nthreads=NTHREADS)
    force_tile(tile)
    # A (M x K) with a wide lda, B (K x N) tight
    dA, keepA = _strided_dev(A, wide_a)
    dC = torch.full((M, N), float("nan"), device="cuda")
    print(f"case tile={tile} wide lda={wide_a} bytes={keepA.numel() * 4}", flush=True)
    binding.gemm_f32_ex(dA, dev(B), dC, 1.0, 0.0, False, False)
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)
    # B stored N x K with a wide ldb
    dBt, keepB = _strided_dev(np.ascontiguousarray(B.T), wide_b)
    dC.fill_(float("nan"))
    print(f"case tile={tile} wide ldb={wide_b} bytes={keepB.numel() * 4}", flush=True)
    binding.gemm_f32_ex(dA, dBt, dC, 1.0, 0.0, False, True)
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)
    del dA, keepA
    # A stored K x M with a wide lda (K rows): offsets (BK - 1) * lda exceed 32 bits
    wide_k = (1 << 30) // 15 + 1000
    dAt, keepAt = _strided_dev(np.ascontiguousarray(A.T), wide_k)
    dC.fill_(float("nan"))
    print(f"case tile={tile} A^T wide lda={wide_k} bytes={keepAt.numel() * 4}", flush=True)
    binding.gemm_f32_ex(dAt, dBt, dC, 1.0, 0.0, True, True)
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)
