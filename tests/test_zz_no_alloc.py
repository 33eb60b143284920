"""The entry point that allocates nothing (gemm_f32_noalloc): its partial products go to a fixed array
in the library's code object instead of an allocated workspace.  Called through the C ABI on raw device
pointers; checked against gemm_f32 (same kernels: the same bits) and against the CPU oracle, on calls in
a row that share the array, a later one smaller than the one before."""
from __future__ import annotations

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_2002_02268_amd import binding, synth  # noqa: E402

from test_gpu_parity import NTHREADS, check_close, dev  # noqa: E402


def _call(fn, M, N, K, dA, dB, dC, transB):
    lda = dA.stride(0)
    ldb = dB.stride(0)
    rc = fn(M, N, K, dA.data_ptr(), lda, dB.data_ptr(), ldb, dC.data_ptr(), dC.stride(0), int(transB))
    assert rc == 0, binding.lib().gemm_f32_strerror(rc).decode()


# (M, N, K, transB): K split (7 MiB of partial products), then a smaller K split, then a split last
# round (13 MiB), then a much smaller K split again, then products that need no scratch at all
SEQUENCE = [(384, 384, 16384, False), (100, 70, 5003, True), (2304, 2304, 2304, False), (128, 128, 8192, False),
            (1000, 1030, 999, False), (300, 270, 515, True)]


def test_noalloc_matches_gemm_f32_and_the_oracle_on_calls_in_a_row():
    lib = binding.lib()
    binding.set_test_hooks()
    lib.gemm_f32_set_stream(None)
    assert binding.gemm_f32_noalloc_scratch_bytes() == 32 << 20
    expect_scratch = ["splitk", "splitk", "tail", "splitk", "strip", ""]
    for idx, (M, N, K, transB) in enumerate(SEQUENCE):
        name = binding.variant_name(M, N, K, transB=transB)
        print(f"noalloc case {idx}: M={M} N={N} K={K} transB={transB} {name}", flush=True)
        assert expect_scratch[idx] in name, name
        A = synth.uniform((M, K), 4000 + idx, synth.TENSOR_A)
        B = synth.uniform((N, K) if transB else (K, N), 4000 + idx, synth.TENSOR_B)
        dA, dB = dev(A), dev(B)
        dC = torch.full((M, N + 3), float("nan"), device="cuda")[:, :N]       # padded rows: ldc = N + 3
        dC_ref = torch.full((M, N + 3), float("nan"), device="cuda")[:, :N]
        _call(lib.gemm_f32_noalloc, M, N, K, dA, dB, dC, transB)
        _call(lib.gemm_f32, M, N, K, dA, dB, dC_ref, transB)
        torch.cuda.synchronize()
        got, want = dC.cpu().numpy(), dC_ref.cpu().numpy()
        assert np.array_equal(got, want), "differs from gemm_f32"
        check_close(got, oracle.gemm_f32(A, B, transB=transB, nthreads=NTHREADS), K)
        # integer operands: exact against the oracle
        Ai = synth.small_ints((M, K), 4100 + idx, synth.TENSOR_A)
        Bi = synth.small_ints((N, K) if transB else (K, N), 4100 + idx, synth.TENSOR_B)
        _call(lib.gemm_f32_noalloc, M, N, K, dev(Ai), dev(Bi), dC, transB)
        assert np.array_equal(dC.cpu().numpy().astype(np.float64), oracle.gemm_f32(Ai, Bi, transB=transB, nthreads=NTHREADS))


def test_noalloc_refuses_a_product_whose_split_needs_more_than_the_array():
    lib = binding.lib()
    binding.set_test_hooks(force_tile=0)                       # the 256 x 256 tile, whatever the cost model prefers
    try:
        lib.gemm_f32_set_stream(None)
        M = N = 4352
        K = 4096
        assert "tail33x7" in binding.variant_name(M, N, K)        # 33 * 7 tiles of 256 x 256 floats: 57.75 MiB
        dA = torch.zeros((M, K), device="cuda")
        dB = torch.zeros((K, N), device="cuda")
        dC = torch.full((M, N), 7.0, device="cuda")
        rc = lib.gemm_f32_noalloc(M, N, K, dA.data_ptr(), K, dB.data_ptr(), N, dC.data_ptr(), N, 0)
        assert rc == -6
        assert "scratch" in lib.gemm_f32_strerror(rc).decode()
        torch.cuda.synchronize()
        assert torch.equal(dC, torch.full((M, N), 7.0, device="cuda")), "something was launched"
        # argument errors are the same as gemm_f32's
        assert lib.gemm_f32_noalloc(8, 8, 8, dA.data_ptr(), 7, dB.data_ptr(), 8, dC.data_ptr(), 8, 0) == -1
        assert lib.gemm_f32_noalloc(8, 8, 8, None, 8, dB.data_ptr(), 8, dC.data_ptr(), 8, 0) == -2
        assert lib.gemm_f32_noalloc(0, 8, 8, None, 8, None, 8, None, 8, 0) == 0
    finally:
        binding.set_test_hooks()
