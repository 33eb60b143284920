"""Seeded synthetic operands for the matrix-product workloads.

This module only produces input values; it holds none of the method's
arithmetic and is the one piece of code that both the GPU tests and the CPU
oracle tests draw from.  The paper's case study (Section 6) multiplies dense
`float` matrices whose contents it never specifies, so the operands are dense
pseudo-random fp32 arrays.

Generator: a counter-based construction, so element (tensor, index) of a given
seed is the same value no matter how or where the array is produced.  The
64-bit counter is scrambled with the SplitMix64 output function (Steele, Lea &
Flood, "Fast splittable pseudorandom number generators", OOPSLA 2014):
    z = key + (index + 1) * 0x9E3779B97F4A7C15
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9
    z = (z ^ (z >> 27)) * 0x94D049BB133111EB
    z =  z ^ (z >> 31)
with key = mix(seed * 2^20 + tensor_id).  The top 24 bits r of z give a uniform
value u = (r + 0.5) / 2^23 - 1 in (-1, 1), exactly representable in fp32.
Standard normals come from Box-Muller on two such streams, evaluated in fp64
and rounded once to fp32.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

TENSOR_A = 0
TENSOR_B = 1
TENSOR_X = 2


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _bits24(seed: int, tensor_id: int, n: int, stream: int = 0) -> np.ndarray:
    """24 random bits per element for flat indices 0..n-1."""
    with np.errstate(over="ignore"):
        key = _mix(np.array([(seed << 20) + (tensor_id << 4) + stream], dtype=np.uint64)
                   * _GOLDEN + _GOLDEN)
        idx = np.arange(1, n + 1, dtype=np.uint64)
        z = _mix(key + idx * _GOLDEN)
    return (z >> np.uint64(40)).astype(np.int64)


def uniform(shape, seed: int, tensor_id: int) -> np.ndarray:
    """fp32 array with entries uniform in (-1, 1)."""
    n = int(np.prod(shape, dtype=np.int64))
    r = _bits24(seed, tensor_id, n)
    u = (r.astype(np.float64) + 0.5) / float(1 << 23) - 1.0
    return u.astype(np.float32).reshape(shape)


def normal(shape, seed: int, tensor_id: int) -> np.ndarray:
    """fp32 array with standard-normal entries (Box-Muller in fp64)."""
    n = int(np.prod(shape, dtype=np.int64))
    r1 = _bits24(seed, tensor_id, n, stream=1).astype(np.float64)
    r2 = _bits24(seed, tensor_id, n, stream=2).astype(np.float64)
    u1 = (r1 + 0.5) / float(1 << 24)          # in (0, 1): log is finite
    u2 = (r2 + 0.5) / float(1 << 24)
    g = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return g.astype(np.float32).reshape(shape)


def small_ints(shape, seed: int, tensor_id: int, lo: int = -2, hi: int = 2) -> np.ndarray:
    """fp32 array of integers in [lo, hi]; products and sums of these are exact in fp32
    as long as K * max(|lo|,|hi|)^2 < 2^24."""
    n = int(np.prod(shape, dtype=np.int64))
    r = _bits24(seed, tensor_id, n, stream=3)
    return (lo + r % (hi - lo + 1)).astype(np.float32).reshape(shape)


def signs(n: int, seed: int, tensor_id: int = TENSOR_X) -> np.ndarray:
    """fp64 vector of +-1 (probe vector for the matrix-vector associativity check)."""
    r = _bits24(seed, tensor_id, n, stream=4)
    return np.where(r & 1, 1.0, -1.0)


# The five workloads: name -> description.  `dist` is the value distribution,
# `transB` says B is stored N x K, `packed` adds a second run on the re-laid-out B.
WORKLOADS = {
    "square1024": dict(batch=0, M=1024, N=1024, K=1024, dist="uniform", seed=0, transB=False),
    "ragged": dict(batch=0, M=1000, N=1030, K=999, dist="uniform", seed=1, transB=False),
    "square4096": dict(batch=0, M=4096, N=4096, K=4096, dist="uniform", seed=2, transB=False),
    "transb2048": dict(batch=0, M=2048, N=2048, K=2048, dist="normal", seed=3, transB=True),
    "batched64": dict(batch=4096, M=64, N=64, K=64, dist="uniform", seed=4, transB=False),
    # one short dimension: 16 flop per byte of the long operand, bound by streaming it (268 MB) once
    "skinny8192": dict(batch=0, M=8192, N=32, K=8192, dist="uniform", seed=5, transB=False),
    "wide8192": dict(batch=0, M=32, N=8192, K=8192, dist="uniform", seed=6, transB=True),
}


def make_operands(name: str, dist: str | None = None):
    """Host fp32 operands (A, B) of a named workload, tight strides.

    A is (M,K) or (batch,M,K); B is (K,N), (N,K) when transB, with a leading
    batch axis for the batched workload.
    """
    w = WORKLOADS[name]
    gen = {"uniform": uniform, "normal": normal, "ints": small_ints}[dist or w["dist"]]
    M, N, K = w["M"], w["N"], w["K"]
    bshape = (N, K) if w["transB"] else (K, N)
    ashape = (M, K)
    if w["batch"]:
        ashape = (w["batch"],) + ashape
        bshape = (w["batch"],) + bshape
    return gen(ashape, w["seed"], TENSOR_A), gen(bshape, w["seed"], TENSOR_B)
