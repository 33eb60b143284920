"""GPU parity of every level of the optimisation ladder against the CPU oracle."""
from __future__ import annotations

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
import workload_refs  # noqa: E402
from paper_2002_02268_amd import binding, synth  # noqa: E402

from test_gpu_parity import NTHREADS, check_close, dev, padded_dev  # noqa: E402

SHAPES = [(1, 1, 1), (33, 65, 17), (130, 257, 70), (300, 140, 129), (64, 64, 64)]


@pytest.mark.parametrize("level", range(7))
def test_ladder_level_matches_oracle(level):
    """Several tiles and ragged tails for every level; padded strides with NaN padding."""
    for idx, (M, N, K) in enumerate(SHAPES):
        print(f"ladder level={level} M={M} N={N} K={K}", flush=True)
        A = synth.uniform((M, K), 90 + idx, synth.TENSOR_A)
        B = synth.uniform((K, N), 90 + idx, synth.TENSOR_B)
        ref = oracle.gemm_f32(A, B, nthreads=NTHREADS)
        dA, _ = padded_dev(A, 3)
        dB, _ = padded_dev(B, 5)
        dC, bufC = padded_dev(np.full((M, N), np.nan, np.float32), 2)
        dBp = torch.full((binding.pack_b_size(N, K) // 4,), float("nan"), device="cuda")
        binding.pack_b(dB, dBp)
        binding.gemm_f32_ladder(level, dA, dB, dC, dBp)
        whole = bufC.cpu().numpy()
        check_close(whole[:, :N], ref, K)
        assert np.isnan(whole[:, N:]).all()


@pytest.mark.parametrize("level", range(7))
def test_ladder_level_integer_bit_exact(level):
    M, N, K = 257, 200, 130
    A = synth.small_ints((M, K), 95, synth.TENSOR_A)
    B = synth.small_ints((K, N), 95, synth.TENSOR_B)
    ref = oracle.gemm_f32(A, B, nthreads=NTHREADS)
    dB = dev(B)
    dBp = torch.empty(binding.pack_b_size(N, K) // 4, device="cuda")
    binding.pack_b(dB, dBp)
    dC = torch.full((M, N), float("nan"), device="cuda")
    binding.gemm_f32_ladder(level, dev(A), dB, dC, dBp)
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)


@pytest.mark.parametrize("name", ["square1024", "square4096"])
def test_ladder_levels_match_the_oracle_on_both_square_workloads(name):
    """The two sizes the ladder is timed at: every element of every level against the oracle's fp64
    product (computed once per size and shared with the product's own parity test)."""
    w = synth.WORKLOADS[name]
    A, B = workload_refs.operands(name)
    ref = workload_refs.reference(name)
    dA, dB = dev(A), dev(B)
    dBp = torch.empty(binding.pack_b_size(w["N"], w["K"]) // 4, device="cuda")
    binding.pack_b(dB, dBp)
    for level in range(7):
        print(f"ladder {name} level={level}", flush=True)
        dC = torch.full((w["M"], w["N"]), float("nan"), device="cuda")
        binding.gemm_f32_ladder(level, dA, dB, dC, dBp)
        check_close(dC.cpu().numpy(), ref, w["K"])
