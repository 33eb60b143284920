"""Calls that use the workspace (a split K, a split last round) running at the same time on two streams
of equal priority, from one host thread and from two: every stream has a workspace of its own, so the
results stay exact.  Integer-valued operands, compared bit for bit with the CPU oracle."""
from __future__ import annotations

import threading

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_2002_02268_amd import binding, synth  # noqa: E402

from test_gpu_parity import NTHREADS, dev  # noqa: E402

# stream 0: K split into 32 ranges (a 12 us product, launched many times);
# stream 1: 68 tiles of the last round split into 3 ranges each (a 190 us product)
CASES = [(128, 128, 8192, False, 40), (2304, 2304, 2304, False, 6)]


def _operands(idx, M, N, K, transB, rep):
    A = synth.small_ints((M, K), 5000 + 10 * idx + rep, synth.TENSOR_A)
    B = synth.small_ints((N, K) if transB else (K, N), 5000 + 10 * idx + rep, synth.TENSOR_B)
    return A, B


def _prepare():
    binding.set_test_hooks()
    work = []
    for idx, (M, N, K, transB, launches) in enumerate(CASES):
        name = binding.variant_name(M, N, K, transB=transB)
        assert ("splitk" in name) if idx == 0 else ("/tail" in name), name
        sets = []
        for rep in range(2):                       # two operand sets per stream, used alternately
            A, B = _operands(idx, M, N, K, transB, rep)
            sets.append((dev(A), dev(B), oracle.gemm_f32(A, B, transB=transB, nthreads=NTHREADS)))
        outs = [torch.full((M, N), float("nan"), device="cuda") for _ in range(launches)]
        work.append((transB, sets, outs))
    torch.cuda.synchronize()
    return work


def _check(work):
    torch.cuda.synchronize()
    for transB, sets, outs in work:
        for i, dC in enumerate(outs):
            assert np.array_equal(dC.cpu().numpy().astype(np.float64), sets[i % 2][2]), f"launch {i}"


def test_workspace_users_on_two_streams_from_one_thread():
    work = _prepare()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    most = max(len(w[2]) for w in work)
    for i in range(most):                          # interleaved: both streams always have work queued
        for s, (transB, sets, outs) in zip(streams, work):
            per = len(outs) / most                 # the short product is launched more often
            for j in range(int(i * per), int((i + 1) * per)):
                with torch.cuda.stream(s):
                    binding.gemm_f32(sets[j % 2][0], sets[j % 2][1], outs[j], transB=transB)
    _check(work)


def test_workspace_users_on_two_streams_from_two_threads():
    work = _prepare()
    errors = []

    def run(transB, sets, outs):
        try:
            s = torch.cuda.Stream()
            with torch.cuda.stream(s):
                for j, dC in enumerate(outs):
                    binding.gemm_f32(sets[j % 2][0], sets[j % 2][1], dC, transB=transB)
            s.synchronize()
        except Exception as e:                     # pragma: no cover
            errors.append(e)

    threads = [threading.Thread(target=run, args=w) for w in work]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    _check(work)


def test_reserved_workspace_is_used_and_shutdown_releases_it():
    binding.set_test_hooks()
    M, N, K = 128, 128, 8192
    A, B = _operands(7, M, N, K, False, 0)
    ref = oracle.gemm_f32(A, B, nthreads=NTHREADS)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        binding.gemm_f32_reserve_workspace(64 << 20)
        dC = torch.full((M, N), float("nan"), device="cuda")
        binding.gemm_f32(dev(A), dev(B), dC)
    s.synchronize()
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)
    assert binding.lib().gemm_f32_reserve_workspace((256 << 20) + 1) == -1
    torch.cuda.synchronize()
    binding.lib().gemm_f32_shutdown()
    with torch.cuda.stream(s):
        dC.fill_(float("nan"))
        binding.gemm_f32(dev(A), dev(B), dC)
    s.synchronize()
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)
