"""Full-output oracle references of the benchmark workloads, computed once per test process.

The fp64 triple loop costs about 22 s at 4096^3 and 3 s at 2048^3 on 16 threads, so the tests that
need the same reference (the product itself, its packed form, the seven ladder levels) share it.
Everything here comes from `oracle/` and the seeded generator; nothing from the HIP library."""
from __future__ import annotations

import functools
import os

import oracle
from paper_2002_02268_amd import synth

NTHREADS = min(16, os.cpu_count() or 1)


@functools.lru_cache(maxsize=None)
def operands(name: str, dist=None):
    """(A, B) of a workload as host arrays (B as the workload stores it)."""
    return synth.make_operands(name, dist=dist)


@functools.lru_cache(maxsize=None)
def reference(name: str, dist=None):
    """The oracle's fp64 C of a whole workload."""
    w = synth.WORKLOADS[name]
    A, B = operands(name, dist)
    print(f"oracle: full reference of {name} dist={dist}", flush=True)
    return oracle.gemm_f32(A, B, transB=w["transB"], nthreads=NTHREADS)
