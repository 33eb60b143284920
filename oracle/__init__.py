"""CPU oracle for the fp32 matrix product -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``gemm_oracle.c`` (plain C, fp64 accumulation, the
definition of Section 6.1 / 6.3 of the paper written out as a triple loop).
Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package; the GPU library never does, and the two share no code.

All arrays are host numpy arrays.  Inputs are float32, results are float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gemm_oracle.c")
_SRC2 = os.path.join(_HERE, "binomial_oracle.c")
_SRC3 = os.path.join(_HERE, "gemm_ex_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_gemm.so")

_i64 = ctypes.c_int64
_fp = ctypes.POINTER(ctypes.c_float)
_dp = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP only splits independent rows)."""
    newest = max(os.path.getmtime(f) for f in (_SRC, _SRC2, _SRC3))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp",
               "-ffp-contract=off", "-o", _LIB, _SRC, _SRC2, _SRC3]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_gemm_f32.argtypes = [_i64, _i64, _i64, _fp, _i64, _fp, _i64, _dp, _i64,
                                        ctypes.c_int, ctypes.c_int]
        lib.oracle_gemm_f32.restype = ctypes.c_int
        lib.oracle_gemm_f32_batched.argtypes = [_i64, _i64, _i64, _i64, _fp, _i64, _i64,
                                                _fp, _i64, _i64, _dp, _i64, _i64,
                                                ctypes.c_int, ctypes.c_int]
        lib.oracle_gemm_f32_batched.restype = ctypes.c_int
        lib.oracle_pack_b.argtypes = [_i64, _i64, _fp, _i64, ctypes.c_int, _i64, _fp]
        lib.oracle_pack_b.restype = ctypes.c_int
        lib.oracle_gemm_f32_packed.argtypes = [_i64, _i64, _i64, _fp, _i64, _fp, _i64, _dp, _i64,
                                               ctypes.c_int]
        lib.oracle_gemm_f32_packed.restype = ctypes.c_int
        lib.oracle_binomial3x3_f32.argtypes = [_i64, _i64, _fp, _i64, _dp, _i64]
        lib.oracle_binomial3x3_f32.restype = ctypes.c_int
        lib.oracle_gemm_f32_ex.argtypes = [_i64, _i64, _i64, ctypes.c_float, _fp, _i64, ctypes.c_int,
                                           _fp, _i64, ctypes.c_int, ctypes.c_float, _fp, _i64,
                                           _dp, _i64, ctypes.c_int]
        lib.oracle_gemm_f32_ex.restype = ctypes.c_int
        lib.oracle_threads_used.argtypes = [ctypes.c_int]
        lib.oracle_threads_used.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f32_2d(x: np.ndarray, name: str) -> np.ndarray:
    if x.dtype != np.float32 or x.ndim != 2:
        raise TypeError(f"{name} must be a 2-D float32 array")
    if x.size == 0:
        return x
    if x.shape[1] > 1 and x.strides[1] != 4:
        raise ValueError(f"{name} must have unit column stride")
    if x.shape[0] > 1 and (x.strides[0] % 4 != 0 or x.strides[0] < 4 * x.shape[1]):
        raise ValueError(f"{name} has an unsupported row stride")
    return x


def _ld(x: np.ndarray) -> int:
    """Leading dimension in elements of a 2-D array with unit column stride."""
    if x.size > 0 and x.shape[0] > 1:
        return max(x.strides[0] // x.itemsize, 1)
    return max(x.shape[1], 1)


def _ptr(x: np.ndarray, ty):
    return x.ctypes.data_as(ty)


def threads_used(nthreads: int) -> int:
    return int(_load().oracle_threads_used(int(nthreads)))


def gemm_f32(A: np.ndarray, B: np.ndarray, transB: bool = False, nthreads: int = 1) -> np.ndarray:
    """C = A @ op(B) in float64; A is (M,K); B is (K,N), or (N,K) when transB.

    Row-strided views are accepted (the row stride becomes lda / ldb).
    """
    A = _f32_2d(A, "A")
    B = _f32_2d(B, "B")
    M, K = A.shape
    if transB:
        N, Kb = B.shape
    else:
        Kb, N = B.shape
    if Kb != K:
        raise ValueError("inner dimensions differ")
    C = np.full((M, N), np.nan, dtype=np.float64)
    rc = _load().oracle_gemm_f32(M, N, K, _ptr(A, _fp), _ld(A), _ptr(B, _fp), _ld(B),
                                 _ptr(C, _dp), max(N, 1), int(bool(transB)), int(nthreads))
    if rc != 0:
        raise ValueError(f"oracle_gemm_f32 rejected its arguments (rc={rc})")
    return C


def gemm_f32_batched(A: np.ndarray, B: np.ndarray, transB: bool = False,
                     nthreads: int = 1) -> np.ndarray:
    """Independent products over a leading batch axis; contiguous (batch, r, c) arrays."""
    if A.dtype != np.float32 or B.dtype != np.float32 or A.ndim != 3 or B.ndim != 3:
        raise TypeError("A and B must be 3-D float32 arrays")
    A = np.ascontiguousarray(A)
    B = np.ascontiguousarray(B)
    batch, M, K = A.shape
    if B.shape[0] != batch:
        raise ValueError("batch sizes differ")
    if transB:
        N, Kb = B.shape[1:]
    else:
        Kb, N = B.shape[1:]
    if Kb != K:
        raise ValueError("inner dimensions differ")
    C = np.full((batch, M, N), np.nan, dtype=np.float64)
    rc = _load().oracle_gemm_f32_batched(batch, M, N, K,
                                         _ptr(A, _fp), max(K, 1), M * K,
                                         _ptr(B, _fp), max(B.shape[2], 1), B.shape[1] * B.shape[2],
                                         _ptr(C, _dp), max(N, 1), M * N,
                                         int(bool(transB)), int(nthreads))
    if rc != 0:
        raise ValueError(f"oracle_gemm_f32_batched rejected its arguments (rc={rc})")
    return C


def pack_b(B: np.ndarray, P: int, transB: bool = False) -> np.ndarray:
    """packedB of shape (ceil(N/P), K, P), ragged last panel zero-filled."""
    B = _f32_2d(B, "B")
    if transB:
        N, K = B.shape
    else:
        K, N = B.shape
    panels = (N + P - 1) // P
    Bp = np.full((panels, K, P), np.nan, dtype=np.float32)
    rc = _load().oracle_pack_b(N, K, _ptr(B, _fp), _ld(B), int(bool(transB)), int(P), _ptr(Bp, _fp))
    if rc != 0:
        raise ValueError(f"oracle_pack_b rejected its arguments (rc={rc})")
    return Bp


def gemm_f32_packed(A: np.ndarray, Bp: np.ndarray, N: int, nthreads: int = 1) -> np.ndarray:
    """C = A @ B where B is given as packedB (panels, K, P)."""
    A = _f32_2d(A, "A")
    if Bp.dtype != np.float32 or Bp.ndim != 3:
        raise TypeError("Bp must be a 3-D float32 array")
    Bp = np.ascontiguousarray(Bp)
    M, K = A.shape
    panels, Kb, P = Bp.shape
    if Kb != K or panels != (N + P - 1) // P:
        raise ValueError("packed operand does not match (N, K)")
    C = np.full((M, N), np.nan, dtype=np.float64)
    rc = _load().oracle_gemm_f32_packed(M, N, K, _ptr(A, _fp), _ld(A), _ptr(Bp, _fp), int(P),
                                        _ptr(C, _dp), max(N, 1), int(nthreads))
    if rc != 0:
        raise ValueError(f"oracle_gemm_f32_packed rejected its arguments (rc={rc})")
    return C


def binomial3x3_f32(img: np.ndarray) -> np.ndarray:
    """3x3 binomial filter (weights 1-2-1 x 1-2-1, /16, repeat-edge) of a 2-D float32 image, in float64.
    Row-strided views are accepted."""
    img = _f32_2d(img, "img")
    H, W = img.shape
    out = np.full((H, W), np.nan, dtype=np.float64)
    rc = _load().oracle_binomial3x3_f32(H, W, _ptr(img, _fp), _ld(img), _ptr(out, _dp), max(W, 1))
    if rc != 0:
        raise ValueError(f"oracle_binomial3x3_f32 rejected its arguments (rc={rc})")
    return out


def gemm_f32_ex(A: np.ndarray, B: np.ndarray, C0: np.ndarray | None = None, alpha: float = 1.0,
                beta: float = 0.0, transA: bool = False, transB: bool = False,
                nthreads: int = 1) -> np.ndarray:
    """alpha * op(A) @ op(B) + beta * C0 in float64.  A is (M,K), or (K,M) when transA; B is (K,N),
    or (N,K) when transB; C0 (float32, (M,N)) is read only when beta != 0."""
    A = _f32_2d(A, "A")
    B = _f32_2d(B, "B")
    K, M = (A.shape if transA else A.shape[::-1])
    Kb, N = (B.shape[::-1] if transB else B.shape)
    if Kb != K:
        raise ValueError("inner dimensions differ")
    if C0 is not None:
        C0 = _f32_2d(C0, "C0")
        if C0.shape != (M, N):
            raise ValueError("C0 has the wrong shape")
    elif beta != 0.0:
        raise ValueError("beta != 0 needs C0")
    C = np.full((M, N), np.nan, dtype=np.float64)
    rc = _load().oracle_gemm_f32_ex(M, N, K, float(alpha), _ptr(A, _fp), _ld(A), int(bool(transA)),
                                    _ptr(B, _fp), _ld(B), int(bool(transB)), float(beta),
                                    _ptr(C0, _fp) if C0 is not None else None,
                                    _ld(C0) if C0 is not None else max(N, 1),
                                    _ptr(C, _dp), max(N, 1), int(nthreads))
    if rc != 0:
        raise ValueError(f"oracle_gemm_f32_ex rejected its arguments (rc={rc})")
    return C
