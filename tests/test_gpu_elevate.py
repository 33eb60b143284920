"""A schedule produced by the strategy layer runs the product on the GPU (gemm_f32_scheduled, through
the C ABI) and is checked against the CPU oracle like any other path: strategy -> scheduled loop
nest -> kernel configuration -> kernel."""
from __future__ import annotations

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_2002_02268_amd import binding as b, synth  # noqa: E402

from test_gpu_parity import NTHREADS, check_close, dev  # noqa: E402


def schedule_text(bm, bn, bk, split, M, N, K):
    """A strategy for a tile shape of the caller's choice, in the form the library writes its own:
    cover the ragged edges, block every axis, reorder into grid / waves / slab / steps / register
    block / instruction, decide every loop, turn the innermost block into the matrix instruction."""
    k_range = -(-(-(-K // split)) // bk) * bk
    blocks = {"M": [(bm, "grid"), (bm // 2, "wave"), (32, "unroll")],
              "N": [(bn, "grid"), (bn // 2, "wave"), (32, "unroll")],
              "K": [(k_range, "grid"), (bk, "slab"), (2, "step")]}
    text, loops, pos = "(seq", [], 0          # loops: (axis, role) in nest order
    for ax, extent in (("M", M), ("N", N), ("K", K)):
        first = blocks[ax][0][0]
        if extent % first:
            text += f" (bodyN {pos} (cover {ax} {first}))"
            extent = -(-extent // first) * first
        for n, role in blocks[ax]:
            if extent > n:
                text += f" (bodyN {pos} (split {ax} {n}))"
                loops.append((ax, role))
                pos += 1
                extent = n
        loops.append((ax, "seq"))
        pos += 1
    order = ["grid", "wave", "slab", "step", "unroll", "seq"]
    perm = [i for role in order for ax in "MNK" for i, l in enumerate(loops) if l == (ax, role)]
    text += " (reorder " + " ".join(map(str, perm)) + ")"
    for newpos, i in enumerate(perm):
        if loops[i][1] in ("grid", "wave", "slab", "unroll"):
            text += f" (bodyN {newpos} (mark {loops[i][1]}))"
    return text + " (topDown mfma))"


CASES = [
    # (M, N, K, transB, tile or None for the library's own strategy, split)
    (1024, 1024, 1024, False, None, 1),
    (1000, 1030, 999, False, None, 1),
    (1000, 1030, 999, True, (128, 128, 16), 1),
    (700, 900, 520, False, (256, 128, 16), 1),
    (700, 900, 520, True, (128, 256, 16), 1),
    (300, 200, 4096, False, (64, 64, 32), 4),
    (128, 128, 8192, False, None, 1),
    (520, 260, 300, False, (256, 256, 16), 1),
    (64, 64, 64, False, (64, 64, 64), 1),
    (2048, 32, 1500, False, None, 1),        # the library's choice here: 32 x 32 blocks whose waves share the slabs
]


@pytest.mark.parametrize("M,N,K,transB,tile,split", CASES)
def test_scheduled_product_matches_the_oracle(M, N, K, transB, tile, split):
    text = b.elevate_default_strategy(M, N, K) if tile is None else schedule_text(*tile, split, M, N, K)
    code, sched, nest = b.elevate_schedule_gemm(M, N, K, text)
    print(f"case M={M} N={N} K={K} transB={transB} schedule={sched.as_dict()}", flush=True)
    assert code == 0, (text, nest)
    if tile is not None:
        assert (sched.bm, sched.bn, sched.bk, sched.split_k) == (*tile, split)
    A = synth.uniform((M, K), 900, synth.TENSOR_A)
    B = synth.uniform((N, K) if transB else (K, N), 900, synth.TENSOR_B)
    ref = oracle.gemm_f32(A, B, transB=transB, nthreads=NTHREADS)
    dC = torch.full((M, N), float("nan"), device="cuda")
    b.gemm_f32_scheduled(sched, dev(A), dev(B), dC, transB=transB)
    check_close(dC.cpu().numpy(), ref, K)
    # integer operands: exact whatever the schedule
    Ai = synth.small_ints((M, K), 901, synth.TENSOR_A)
    Bi = synth.small_ints((N, K) if transB else (K, N), 901, synth.TENSOR_B)
    b.gemm_f32_scheduled(sched, dev(Ai), dev(Bi), dC, transB=transB)
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), oracle.gemm_f32(Ai, Bi, transB=transB, nthreads=NTHREADS))


def test_default_schedule_runs_the_same_kernel_as_the_plain_entry_point():
    for (M, N, K) in [(1024, 1024, 1024), (1536, 1536, 1536), (96, 80, 4000)]:
        code, sched, _ = b.elevate_schedule_gemm(M, N, K, b.elevate_default_strategy(M, N, K))
        assert code == 0
        A = torch.rand(M, K, device="cuda")
        B = torch.rand(K, N, device="cuda")
        C1 = torch.empty(M, N, device="cuda")
        C2 = torch.empty(M, N, device="cuda")
        b.gemm_f32(A, B, C1)
        b.gemm_f32_scheduled(sched, A, B, C2)
        assert torch.equal(C1, C2)


def test_filter_scheduled_by_a_strategy_matches_the_oracle():
    """Section 5 end to end: the naive filter, rewritten by topDown(separateDot) and a storage choice,
    selects one of the three kernels; each result is checked against the nine-tap oracle."""
    separate = "(topDown (separateDot weights2d weightsH weightsV))"
    strategies = {"id": 0, f"(seq {separate} (topDown (storeRows image)))": 1,
                  f"(seq {separate} (topDown (storeRows line)))": 2}
    img = synth.uniform((300, 517), 950, synth.TENSOR_A)
    ints = synth.small_ints((300, 517), 951, synth.TENSOR_A, -50, 50)
    for text, want in strategies.items():
        code, form, prog = b.elevate_schedule_filter(text)
        assert (code, form) == (0, want), prog
        for image, exact in ((img, False), (ints, True)):
            out = torch.full((300, 517), float("nan"), device="cuda")
            tmp = torch.empty((300, 517), device="cuda")
            b.binomial3x3_f32_variant(form, dev(image), out, tmp)
            got = out.cpu().numpy().astype(np.float64)
            ref = oracle.binomial3x3_f32(image)
            assert np.array_equal(got, ref) if exact else np.max(np.abs(got - ref)) <= 1e-6
