"""GPU parity of gemm_f32_ex on seeded random shapes, layouts, scalings, row paddings and tile
choices (the dispatch's own and forced ones) against the general-form CPU oracle.

Integer-valued operands in {-3..3}, integer or half-integer alpha and beta, C_old in {-5..5}:
every partial sum is an integer (or a multiple of 1/2) far below 2^24, so any summation order is
exact and the comparison is bit for bit.  The shape classes aim at the dispatch's special cases:
one short dimension (the 32-wide tiles and the tile whose waves share the slabs), small outputs
with long K (K splits), tile counts a little above a multiple of 256 (split last round, with and
without 32 x 32 blocks), plain mid-size products with ragged edges, and outputs of several hundred to a
thousand tiles with a short K, where workgroups share compute units and their epilogues overlap."""
from __future__ import annotations

import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_2002_02268_amd import binding, synth  # noqa: E402

from test_gpu_parity import NTHREADS, TILES, padded_dev  # noqa: E402

TENSOR_C = 2
CASES_PER_CLASS = 24


def _draw(rng, cls):
    r = lambda lo, hi: int(rng.integers(lo, hi + 1))  # noqa: E731
    if cls == "short_m":
        return r(1, 40), r(1, 5000), r(1, 3000)
    if cls == "short_n":
        return r(1, 5000), r(1, 40), r(1, 3000)
    if cls == "long_k":
        return r(1, 300), r(1, 300), r(2000, 20000)
    if cls == "second_round":
        return r(1000, 1300), r(1000, 1300), r(1, 700)
    if cls == "co_resident":
        return r(1500, 4000), r(1500, 4000), r(20, 900)
    return r(1, 1500), r(1, 1500), r(1, 900)


@pytest.mark.parametrize("cls", ["short_m", "short_n", "long_k", "second_round", "plain", "co_resident"])
def test_random_shapes_bit_exact(cls):
    rng = np.random.default_rng({"short_m": 11, "short_n": 12, "long_k": 13, "second_round": 14, "plain": 15,
                                 "co_resident": 16}[cls])
    tiles = [None, None, None] + list(TILES.values())
    try:
        for idx in range(CASES_PER_CLASS):
            M, N, K = _draw(rng, cls)
            tA, tB = bool(rng.random() < 0.4), bool(rng.random() < 0.5)
            alpha = float(rng.choice([1.0, 1.0, -2.0, 0.5]))
            beta = float(rng.choice([0.0, 0.0, 1.0, -0.5]))
            pa, pb, pc = int(rng.choice([0, 0, 3, 8])), int(rng.choice([0, 0, 1, 4])), int(rng.choice([0, 0, 5]))
            tile = tiles[int(rng.integers(0, len(tiles)))]
            print(f"case {cls}[{idx}] M={M} N={N} K={K} tA={tA} tB={tB} alpha={alpha} beta={beta} "
                  f"pads=({pa},{pb},{pc}) tile={tile}", flush=True)
            A = synth.small_ints((K, M) if tA else (M, K), 9000 + idx, synth.TENSOR_A, lo=-3, hi=3)
            B = synth.small_ints((N, K) if tB else (K, N), 9000 + idx, synth.TENSOR_B, lo=-3, hi=3)
            C0 = synth.small_ints((M, N), 9000 + idx, TENSOR_C, lo=-5, hi=5)
            ref = oracle.gemm_f32_ex(A, B, C0, alpha, beta, tA, tB, nthreads=NTHREADS)
            dA, _ = padded_dev(A, pa)
            dB, _ = padded_dev(B, pb)
            dC, bufC = padded_dev(C0, pc)
            if tile is None:
                binding.set_test_hooks(force_tile=None)
            else:
                binding.set_test_hooks(force_tile=tile)
            binding.gemm_f32_ex(dA, dB, dC, alpha, beta, tA, tB)
            whole = bufC.cpu().numpy()
            assert np.array_equal(whole[:, :N].astype(np.float64), ref)
            assert np.isnan(whole[:, N:]).all(), "ldc padding was written"
    finally:
        binding.set_test_hooks(force_tile=None)


def test_random_batched_shapes_bit_exact():
    """Batched products on seeded random shapes and batch counts, either layout of B, the dispatch's own
    tile and forced ones (small outputs with long K take the tiles whose waves share the slabs, since a
    batched product cannot split K): integer operands, exact against a loop of single oracle products."""
    rng = np.random.default_rng(21)
    tiles = [None, None] + list(TILES.values())
    try:
        for idx in range(30):
            batch = int(rng.integers(2, 40))
            M, N, K = int(rng.integers(1, 300)), int(rng.integers(1, 300)), int(rng.integers(1, 2500))
            tB = bool(rng.random() < 0.5)
            tile = tiles[int(rng.integers(0, len(tiles)))]
            print(f"case batched[{idx}] batch={batch} M={M} N={N} K={K} tB={tB} tile={tile}", flush=True)
            A = synth.small_ints((batch, M, K), 9500 + idx, synth.TENSOR_A, lo=-3, hi=3)
            B = synth.small_ints((batch, N, K) if tB else (batch, K, N), 9500 + idx, synth.TENSOR_B, lo=-3, hi=3)
            ref = oracle.gemm_f32_batched(A, B, transB=tB, nthreads=NTHREADS)
            dC = torch.full((batch, M, N), float("nan"), device="cuda")
            if tile is None:
                binding.set_test_hooks(force_tile=None)
            else:
                binding.set_test_hooks(force_tile=tile)
            binding.gemm_f32_batched(torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda(), dC, transB=tB)
            assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)
    finally:
        binding.set_test_hooks(force_tile=None)


def test_narrow_b_stored_k_by_n_bit_exact():
    """Outputs narrower than a 32-wide tile with B stored K x N (rows of N floats, NaN behind them): for
    N a multiple of 4 the 32-wide tiles load B 16 bytes at a time and mask whole slots, otherwise
    element by element; nothing beyond column N may be read into the sum or written."""
    rng = np.random.default_rng(31)
    tiles = [None, None, TILES["t128x32"], TILES["tq32"], TILES["tq64x32"], TILES["t64"]]
    try:
        for idx in range(48):
            N = int(rng.choice([4, 8, 12, 16, 20, 24, 28, 32, 36, 44, 6, 17, 31, 1, 3]))
            M = int(rng.choice([rng.integers(1, 40), rng.integers(1, 3000), rng.integers(1024, 5000)]))
            K = int(rng.integers(1, 2500))
            tA = bool(rng.random() < 0.3)
            alpha, beta = float(rng.choice([1.0, -2.0, 0.5])), float(rng.choice([0.0, 1.0, -0.5]))
            tile = tiles[int(rng.integers(0, len(tiles)))]
            print(f"case narrow[{idx}] M={M} N={N} K={K} tA={tA} alpha={alpha} beta={beta} tile={tile}", flush=True)
            A = synth.small_ints((K, M) if tA else (M, K), 9700 + idx, synth.TENSOR_A, lo=-3, hi=3)
            B = synth.small_ints((K, N), 9700 + idx, synth.TENSOR_B, lo=-3, hi=3)
            C0 = synth.small_ints((M, N), 9700 + idx, TENSOR_C, lo=-5, hi=5)
            ref = oracle.gemm_f32_ex(A, B, C0, alpha, beta, tA, False, nthreads=NTHREADS)
            dA, _ = padded_dev(A, int(rng.choice([0, 3, 8])))
            dB, _ = padded_dev(B, int(rng.choice([0, 1, 4, 7])))
            dC, bufC = padded_dev(C0, int(rng.choice([0, 5])))
            if tile is None:
                binding.set_test_hooks(force_tile=None)
            else:
                binding.set_test_hooks(force_tile=tile)
            binding.gemm_f32_ex(dA, dB, dC, alpha, beta, tA, False)
            whole = bufC.cpu().numpy()
            assert np.array_equal(whole[:, :N].astype(np.float64), ref)
            assert np.isnan(whole[:, N:]).all(), "ldc padding was written"
    finally:
        binding.set_test_hooks(force_tile=None)


def test_thin_products_vector_unit_kernel_bit_exact():
    """Products with at most 8 rows or columns and both operands stored with k contiguous: the kernel
    that streams the long operand through the vector unit, forced wherever it can run, on ragged row
    counts (waves with fewer than four rows left), K around the 16-byte and 1 KB request sizes, NaN
    behind every row of both operands, alpha / beta, padded C.  Exact on integer operands.  The last
    case is one the dispatch sends there by itself."""
    rng = np.random.default_rng(41)
    binding.set_test_hooks(force_thin=True)
    try:
        for idx in range(40):
            S = int(rng.integers(1, 9))
            big = int(rng.choice([64, 65, 66, 67, 100, 257, 1000, 4099, int(rng.integers(64, 6000))]))
            K = int(rng.choice([1, 2, 3, 4, 5, 255, 256, 257, 511, 512, 513, 1000, 2051, int(rng.integers(1, 6000))]))
            M, N = (S, big) if rng.random() < 0.5 else (big, S)
            alpha, beta = float(rng.choice([1.0, -2.0, 0.5])), float(rng.choice([0.0, 1.0, -0.5]))
            name = binding.variant_name(M, N, K, transB=True)
            print(f"case thin[{idx}] M={M} N={N} K={K} alpha={alpha} beta={beta} {name}", flush=True)
            assert name == f"thin{S}x4/nt", name
            A = synth.small_ints((M, K), 9800 + idx, synth.TENSOR_A, lo=-3, hi=3)
            B = synth.small_ints((N, K), 9800 + idx, synth.TENSOR_B, lo=-3, hi=3)
            C0 = synth.small_ints((M, N), 9800 + idx, TENSOR_C, lo=-5, hi=5)
            ref = oracle.gemm_f32_ex(A, B, C0, alpha, beta, False, True, nthreads=NTHREADS)
            dA, _ = padded_dev(A, int(rng.choice([0, 3, 8])))
            dB, _ = padded_dev(B, int(rng.choice([0, 1, 4, 7])))
            dC, bufC = padded_dev(C0, int(rng.choice([0, 5])))
            binding.gemm_f32_ex(dA, dB, dC, alpha, beta, False, True)
            whole = bufC.cpu().numpy()
            assert np.array_equal(whole[:, :N].astype(np.float64), ref)
            assert np.isnan(whole[:, N:]).all(), "ldc padding was written"
    finally:
        binding.set_test_hooks(force_thin=None)
    M, N, K = 3, 4100, 10300
    assert binding.variant_name(M, N, K, transB=True) == "thin3x4/nt"
    A = synth.small_ints((M, K), 9900, synth.TENSOR_A)
    B = synth.small_ints((N, K), 9900, synth.TENSOR_B)
    ref = oracle.gemm_f32(A, B, transB=True, nthreads=NTHREADS)
    dC = torch.full((M, N), float("nan"), device="cuda")
    binding.gemm_f32(torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda(), dC, transB=True)
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)
    # uniform operands: within the product's tolerance, and the same bits on every launch
    A, B = synth.uniform((M, K), 9901, synth.TENSOR_A), synth.uniform((N, K), 9901, synth.TENSOR_B)
    ref = oracle.gemm_f32(A, B, transB=True, nthreads=NTHREADS)
    outs = []
    for _ in range(3):
        dC = torch.full((M, N), float("nan"), device="cuda")
        binding.gemm_f32(torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda(), dC, transB=True)
        outs.append(dC.cpu().numpy())
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    err = np.abs(outs[0].astype(np.float64) - ref).max()
    assert err <= 1e-3 * (K / 1024.0) ** 0.5, err
