"""ctypes binding for libgemmf32.so: same names as the C ABI in include/gemm_f32.h.

Argument marshalling only.  Tensors are torch CUDA (HIP) tensors used as device
memory; every arithmetic step runs inside the library's kernels.  There is no
fallback: if the built library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgemmf32.so")

_i64 = ctypes.c_int64
_ptr = ctypes.c_void_p

SYMBOLS = {
    "gemm_f32": (ctypes.c_int, [_i64, _i64, _i64, _ptr, _i64, _ptr, _i64, _ptr, _i64, ctypes.c_int]),
    "gemm_f32_batched": (ctypes.c_int, [_i64, _i64, _i64, _i64, _ptr, _i64, _i64, _ptr, _i64, _i64,
                                        _ptr, _i64, _i64, ctypes.c_int]),
    "gemm_f32_ex": (ctypes.c_int, [_i64, _i64, _i64, ctypes.c_float, _ptr, _i64, ctypes.c_int, _ptr, _i64,
                                   ctypes.c_int, ctypes.c_float, _ptr, _i64]),
    "gemm_f32_ex_batched": (ctypes.c_int, [_i64, _i64, _i64, _i64, ctypes.c_float, _ptr, _i64, _i64, ctypes.c_int,
                                           _ptr, _i64, _i64, ctypes.c_int, ctypes.c_float, _ptr, _i64, _i64]),
    "pack_b_panel_width": (_i64, []),
    "pack_b_size": (ctypes.c_size_t, [_i64, _i64]),
    "pack_b": (ctypes.c_int, [_i64, _i64, _ptr, _i64, ctypes.c_int, _ptr]),
    "gemm_f32_packed": (ctypes.c_int, [_i64, _i64, _i64, _ptr, _i64, _ptr, _ptr, _i64]),
    "gemm_f32_set_stream": (ctypes.c_int, [_ptr]),
    "gemm_f32_reserve_workspace": (ctypes.c_int, [ctypes.c_size_t]),
    "gemm_f32_noalloc": (ctypes.c_int, [_i64, _i64, _i64, _ptr, _i64, _ptr, _i64, _ptr, _i64, ctypes.c_int]),
    "gemm_f32_noalloc_scratch_bytes": (ctypes.c_size_t, []),
    "gemm_f32_set_test_hooks": (ctypes.c_int, [_ptr]),
    "gemm_f32_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "gemm_f32_last_hip_error": (ctypes.c_int, []),
    "gemm_f32_shutdown": (None, []),
    "gemm_f32_mfma_rate_probe": (ctypes.c_int, [_i64, _ptr, _ptr]),
    "gemm_f32_variant_name": (ctypes.c_char_p, [_i64, _i64, _i64, _ptr, _i64, _ptr, _i64, _ptr, _i64,
                                                ctypes.c_int]),
    "gemm_f32_ladder_levels": (ctypes.c_int, []),
    "gemm_f32_ladder_name": (ctypes.c_char_p, [ctypes.c_int]),
    "gemm_f32_ladder": (ctypes.c_int, [ctypes.c_int, _i64, _i64, _i64, _ptr, _i64, _ptr, _i64, _ptr, _ptr, _i64]),
    "gemm_f32_ladder_set_stream": (ctypes.c_int, [_ptr]),
    "binomial3x3_f32": (ctypes.c_int, [_i64, _i64, _ptr, _i64, _ptr, _i64]),
    "binomial3x3_f32_set_stream": (ctypes.c_int, [_ptr]),
    "binomial3x3_f32_variant": (ctypes.c_int, [ctypes.c_int, _i64, _i64, _ptr, _i64, _ptr, _i64, _ptr, _i64]),
    "binomial3x3_f32_variants": (ctypes.c_int, []),
    "binomial3x3_f32_variant_name": (ctypes.c_char_p, [ctypes.c_int]),
    "elevate_rewrite": (ctypes.c_int, [ctypes.c_char_p, ctypes.c_char_p, ctypes.c_char_p, ctypes.c_size_t,
                                       ctypes.POINTER(ctypes.c_int), ctypes.c_char_p, ctypes.c_size_t]),
    "elevate_alpha_equal": (ctypes.c_int, [ctypes.c_char_p, ctypes.c_char_p]),
    "elevate_schedule_gemm": (ctypes.c_int, [_i64, _i64, _i64, ctypes.c_char_p, _ptr, ctypes.c_char_p, ctypes.c_size_t]),
    "elevate_schedule_filter": (ctypes.c_int, [ctypes.c_char_p, ctypes.POINTER(ctypes.c_int), ctypes.c_char_p,
                                               ctypes.c_size_t]),
    "elevate_default_strategy": (ctypes.c_int, [_i64, _i64, _i64, ctypes.c_char_p, ctypes.c_size_t]),
    "elevate_dispatch_stats": (None, [ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]),
    "gemm_f32_scheduled": (ctypes.c_int, [_ptr, _i64, _i64, _i64, _ptr, _i64, _ptr, _i64, _ptr, _i64, ctypes.c_int]),
}

_lib = None


class GemmError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"gemm_f32 library error {status}: {message}")
        self.status = status


def lib() -> ctypes.CDLL:
    """The loaded library (built beforehand; build it here only if no build exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build(force=True)
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(handle, name)   # AttributeError if the symbol is missing
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _check(status: int) -> None:
    if status != 0:
        raise GemmError(status, lib().gemm_f32_strerror(status).decode())


def _dev_f32(t, name: str, ndim: int):
    import torch
    if not isinstance(t, torch.Tensor) or t.dtype != torch.float32 or not t.is_cuda:
        raise TypeError(f"{name} must be a float32 tensor on the GPU")
    if t.dim() != ndim:
        raise ValueError(f"{name} must have {ndim} dimensions")
    if t.numel() > 0 and t.shape[-1] > 1 and t.stride(-1) != 1:
        raise ValueError(f"{name} must have unit stride in its last dimension")
    return t


def _ld(t) -> int:
    """Leading dimension (elements) of the last two axes."""
    if t.numel() > 0 and t.shape[-2] > 1:
        return max(int(t.stride(-2)), 1)
    return max(int(t.shape[-1]), 1)


def _use_current_stream(t) -> None:
    import torch
    lib().gemm_f32_set_stream(ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream))


def gemm_f32(A, B, C, transB: bool = False) -> None:
    """C[:] = A @ op(B) on the current torch stream.  A (M,K); B (K,N) or (N,K) if transB; C (M,N).
    Row-strided views are passed through as lda / ldb / ldc."""
    A = _dev_f32(A, "A", 2)
    B = _dev_f32(B, "B", 2)
    C = _dev_f32(C, "C", 2)
    M, K = A.shape
    N = B.shape[0] if transB else B.shape[1]
    if (B.shape[1] if transB else B.shape[0]) != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    _use_current_stream(C)
    _check(lib().gemm_f32(M, N, K, A.data_ptr(), _ld(A), B.data_ptr(), _ld(B), C.data_ptr(), _ld(C),
                          int(bool(transB))))


def gemm_f32_noalloc(A, B, C, transB: bool = False) -> None:
    """gemm_f32 through the entry point that allocates nothing (fixed scratch array)."""
    A = _dev_f32(A, "A", 2)
    B = _dev_f32(B, "B", 2)
    C = _dev_f32(C, "C", 2)
    M, K = A.shape
    N = B.shape[0] if transB else B.shape[1]
    if (B.shape[1] if transB else B.shape[0]) != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    _use_current_stream(C)
    _check(lib().gemm_f32_noalloc(M, N, K, A.data_ptr(), _ld(A), B.data_ptr(), _ld(B), C.data_ptr(), _ld(C),
                                  int(bool(transB))))


def gemm_f32_noalloc_scratch_bytes() -> int:
    return int(lib().gemm_f32_noalloc_scratch_bytes())


def gemm_f32_reserve_workspace(nbytes: int, device=None) -> None:
    """Sizes the workspace of the current torch stream ahead of time."""
    import torch
    lib().gemm_f32_set_stream(ctypes.c_void_p(torch.cuda.current_stream(device).cuda_stream))
    _check(lib().gemm_f32_reserve_workspace(int(nbytes)))


class HookSettings(ctypes.Structure):
    """gemmf32_test_hooks (include/gemm_f32_testing.h)"""
    _fields_ = [("force_tile", ctypes.c_int32), ("force_split", ctypes.c_int32), ("no_tail_split", ctypes.c_int32),
                ("no_quad", ctypes.c_int32), ("no_kshare", ctypes.c_int32), ("no_thin", ctypes.c_int32),
                ("force_thin", ctypes.c_int32), ("no_strip", ctypes.c_int32), ("strip_wait", ctypes.c_int32),
                ("force_strip", ctypes.c_int32), ("strip_rows", ctypes.c_int32)]


_hooks = {}


def set_test_hooks(**changes) -> None:
    """Changes some of the dispatch overrides and leaves the others as they are: force_tile=3,
    no_quad=True, ...; a value of None (or False, or 0 for force_split) switches that override off.
    Without arguments: everything off (production)."""
    if not changes:
        _hooks.clear()
    for key, value in changes.items():
        if key not in dict(HookSettings._fields_):
            raise KeyError(key)
        if value is None or value is False:
            _hooks.pop(key, None)
        else:
            _hooks[key] = int(value)
    h = HookSettings(force_tile=_hooks.get("force_tile", -1), force_split=_hooks.get("force_split", 0),
                  **{k: _hooks.get(k, 0) for k in ("no_tail_split", "no_quad", "no_kshare", "no_thin", "force_thin", "no_strip", "strip_wait", "force_strip", "strip_rows")})
    _check(lib().gemm_f32_set_test_hooks(ctypes.byref(h)))


def gemm_f32_batched(A, B, C, transB: bool = False) -> None:
    """C[b] = A[b] @ op(B[b]) for 3-D tensors with a leading batch axis."""
    A = _dev_f32(A, "A", 3)
    B = _dev_f32(B, "B", 3)
    C = _dev_f32(C, "C", 3)
    batch, M, K = A.shape
    N = B.shape[1] if transB else B.shape[2]
    if B.shape[0] != batch or (B.shape[2] if transB else B.shape[1]) != K or tuple(C.shape) != (batch, M, N):
        raise ValueError("shape mismatch")
    _use_current_stream(C)
    _check(lib().gemm_f32_batched(batch, M, N, K,
                                  A.data_ptr(), _ld(A), int(A.stride(0)),
                                  B.data_ptr(), _ld(B), int(B.stride(0)),
                                  C.data_ptr(), _ld(C), int(C.stride(0)), int(bool(transB))))


def gemm_f32_ex(A, B, C, alpha: float = 1.0, beta: float = 0.0, transA: bool = False, transB: bool = False) -> None:
    """C[:] = alpha * op(A) @ op(B) + beta * C.  A (M,K), or (K,M) if transA; B (K,N), or (N,K) if transB."""
    A = _dev_f32(A, "A", 2)
    B = _dev_f32(B, "B", 2)
    C = _dev_f32(C, "C", 2)
    K, M = (A.shape if transA else A.shape[::-1])
    Kb, N = (B.shape[::-1] if transB else B.shape)
    if Kb != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    _use_current_stream(C)
    _check(lib().gemm_f32_ex(M, N, K, float(alpha), A.data_ptr(), _ld(A), int(bool(transA)), B.data_ptr(), _ld(B),
                             int(bool(transB)), float(beta), C.data_ptr(), _ld(C)))


def gemm_f32_ex_batched(A, B, C, alpha: float = 1.0, beta: float = 0.0, transA: bool = False,
                        transB: bool = False) -> None:
    """Batched general form over a leading batch axis; batch strides are taken from the tensors."""
    A = _dev_f32(A, "A", 3)
    B = _dev_f32(B, "B", 3)
    C = _dev_f32(C, "C", 3)
    batch = A.shape[0]
    K, M = (A.shape[1:] if transA else A.shape[:0:-1])
    Kb, N = (B.shape[:0:-1] if transB else B.shape[1:])
    if B.shape[0] != batch or Kb != K or tuple(C.shape) != (batch, M, N):
        raise ValueError("shape mismatch")
    _use_current_stream(C)
    _check(lib().gemm_f32_ex_batched(batch, M, N, K, float(alpha), A.data_ptr(), _ld(A), int(A.stride(0)),
                                     int(bool(transA)), B.data_ptr(), _ld(B), int(B.stride(0)), int(bool(transB)),
                                     float(beta), C.data_ptr(), _ld(C), int(C.stride(0))))


def gemm_f32_mfma_rate_probe(mfma_per_wave: int, operands, sink) -> None:
    """Launches the matrix-instruction-only kernel (see gemm_f32.h) on the current torch stream."""
    if operands.numel() < 512 or not operands.is_contiguous():
        raise ValueError("operands must hold 512 contiguous floats")
    _dev_f32(operands, "operands", 1)
    _use_current_stream(sink)
    _check(lib().gemm_f32_mfma_rate_probe(int(mfma_per_wave), operands.data_ptr(), sink.data_ptr()))


def pack_b_panel_width() -> int:
    return int(lib().pack_b_panel_width())


def pack_b_size(N: int, K: int) -> int:
    return int(lib().pack_b_size(N, K))


def pack_b(B, Bp, transB: bool = False) -> None:
    """Writes packedB (ceil(N/P), K, P) into the float32 device tensor Bp (at least pack_b_size bytes)."""
    B = _dev_f32(B, "B", 2)
    N, K = (B.shape[0], B.shape[1]) if transB else (B.shape[1], B.shape[0])
    if not Bp.is_cuda or Bp.dtype != B.dtype or not Bp.is_contiguous():
        raise TypeError("Bp must be a contiguous float32 tensor on the GPU")
    if Bp.numel() * 4 < pack_b_size(N, K):
        raise ValueError("Bp is smaller than pack_b_size(N, K)")
    _use_current_stream(Bp)
    _check(lib().pack_b(N, K, B.data_ptr(), _ld(B), int(bool(transB)), Bp.data_ptr()))


def gemm_f32_packed(A, Bp, C) -> None:
    """C[:] = A @ B with B given as the packed buffer written by pack_b for the same (N, K)."""
    A = _dev_f32(A, "A", 2)
    C = _dev_f32(C, "C", 2)
    M, K = A.shape
    N = C.shape[1]
    if C.shape[0] != M:
        raise ValueError("shape mismatch")
    if not Bp.is_cuda or not Bp.is_contiguous() or Bp.numel() * 4 < pack_b_size(N, K):
        raise ValueError("Bp does not hold a packed (N, K) operand")
    _use_current_stream(C)
    _check(lib().gemm_f32_packed(M, N, K, A.data_ptr(), _ld(A), Bp.data_ptr(), C.data_ptr(), _ld(C)))


def variant_name(M: int, N: int, K: int, lda=None, ldb=None, ldc=None, transB: bool = False) -> str:
    lda = lda or max(K, 1)
    ldb = ldb or max(K if transB else N, 1)
    ldc = ldc or max(N, 1)
    return lib().gemm_f32_variant_name(M, N, K, None, lda, None, ldb, None, ldc, int(bool(transB))).decode()


def gemm_f32_ladder_levels() -> int:
    return int(lib().gemm_f32_ladder_levels())


def gemm_f32_ladder_name(level: int) -> str:
    return lib().gemm_f32_ladder_name(int(level)).decode()


def gemm_f32_ladder(level: int, A, B, C, Bp=None) -> None:
    """C[:] = A @ B by ladder level `level` (B row-major K x N; Bp: packed B for levels >= 4)."""
    import torch
    A = _dev_f32(A, "A", 2)
    B = _dev_f32(B, "B", 2)
    C = _dev_f32(C, "C", 2)
    M, K = A.shape
    N = B.shape[1]
    if B.shape[0] != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    if level >= 4 and (Bp is None or Bp.numel() * 4 < pack_b_size(N, K)):
        raise ValueError("levels 4-6 need the packed operand from pack_b")
    stream = ctypes.c_void_p(torch.cuda.current_stream(C.device).cuda_stream)
    lib().gemm_f32_ladder_set_stream(stream)
    _check(lib().gemm_f32_ladder(int(level), M, N, K, A.data_ptr(), _ld(A), B.data_ptr(), _ld(B),
                                 Bp.data_ptr() if Bp is not None else None, C.data_ptr(), _ld(C)))


def binomial3x3_f32(img, out) -> None:
    """out[:] = 3x3 binomial filter of img (2-D float32 device tensors of equal shape; row strides allowed)."""
    import torch
    img = _dev_f32(img, "img", 2)
    out = _dev_f32(out, "out", 2)
    if tuple(img.shape) != tuple(out.shape):
        raise ValueError("shape mismatch")
    H, W = img.shape
    lib().binomial3x3_f32_set_stream(ctypes.c_void_p(torch.cuda.current_stream(out.device).cuda_stream))
    _check(lib().binomial3x3_f32(H, W, img.data_ptr(), _ld(img), out.data_ptr(), _ld(out)))


def binomial3x3_f32_variants() -> int:
    return int(lib().binomial3x3_f32_variants())


def binomial3x3_f32_variant_name(variant: int) -> str:
    return lib().binomial3x3_f32_variant_name(int(variant)).decode()


def binomial3x3_f32_variant(variant: int, img, out, tmp=None) -> None:
    """out[:] = 3x3 binomial filter of img by form `variant` (0 naive, 1 separated: needs tmp, 2 scanline)."""
    import torch
    img = _dev_f32(img, "img", 2)
    out = _dev_f32(out, "out", 2)
    if tuple(img.shape) != tuple(out.shape):
        raise ValueError("shape mismatch")
    if tmp is not None:
        tmp = _dev_f32(tmp, "tmp", 2)
        if tuple(tmp.shape) != tuple(img.shape):
            raise ValueError("tmp must have the shape of the image")
    H, W = img.shape
    lib().binomial3x3_f32_set_stream(ctypes.c_void_p(torch.cuda.current_stream(out.device).cuda_stream))
    _check(lib().binomial3x3_f32_variant(int(variant), H, W, img.data_ptr(), _ld(img), out.data_ptr(), _ld(out),
                                         tmp.data_ptr() if tmp is not None else None,
                                         _ld(tmp) if tmp is not None else max(W, 1)))


# ---- strategy layer (include/elevate.h) -------------------------------------------------------------

class Schedule(ctypes.Structure):
    """gemmf32_schedule"""
    _fields_ = [("bm", ctypes.c_int32), ("bn", ctypes.c_int32), ("bk", ctypes.c_int32),
                ("waves_m", ctypes.c_int32), ("waves_n", ctypes.c_int32),
                ("wave_m", ctypes.c_int32), ("wave_n", ctypes.c_int32), ("split_k", ctypes.c_int32),
                ("tiles_m", ctypes.c_int64), ("tiles_n", ctypes.c_int64), ("k_range", ctypes.c_int64),
                ("waves_k", ctypes.c_int32)]

    def as_dict(self):
        return {name: int(getattr(self, name)) for name, _ in self._fields_}


ELEVATE_OK, ELEVATE_FAILED, ELEVATE_EPARSE, ELEVATE_ENULL = 0, 1, -1, -2
ELEVATE_ELIMIT, ELEVATE_ELOWER, ELEVATE_ENOKERNEL = -6, -7, -8


def elevate_rewrite(strategy: str, program: str, trace: bool = False):
    """Applies a strategy to a program (both s-expressions).  Returns (code, text, steps[, trace])."""
    out = ctypes.create_string_buffer(1 << 16)
    steps = ctypes.c_int(0)
    tbuf = ctypes.create_string_buffer(1 << 20) if trace else None
    rc = lib().elevate_rewrite(strategy.encode(), program.encode(), out, len(out), ctypes.byref(steps), tbuf,
                               len(tbuf) if trace else 0)
    res = (rc, out.value.decode(), steps.value)
    return res + (tbuf.value.decode(),) if trace else res


def elevate_alpha_equal(a: str, b: str) -> int:
    return int(lib().elevate_alpha_equal(a.encode(), b.encode()))


def elevate_schedule_gemm(M: int, N: int, K: int, strategy: str):
    """Schedules the product's loop nest with a strategy and lowers it.  Returns (code, Schedule, nest text)."""
    sched = Schedule()
    nest = ctypes.create_string_buffer(1 << 14)
    rc = lib().elevate_schedule_gemm(M, N, K, strategy.encode(), ctypes.byref(sched), nest, len(nest))
    return rc, sched, nest.value.decode()


def elevate_schedule_filter(strategy: str):
    """Rewrites the naive binomial filter with a strategy.  Returns (code, form, program text)."""
    form = ctypes.c_int(-1)
    buf = ctypes.create_string_buffer(1 << 12)
    rc = lib().elevate_schedule_filter(strategy.encode(), ctypes.byref(form), buf, len(buf))
    return rc, form.value, buf.value.decode()


def elevate_default_strategy(M: int, N: int, K: int) -> str:
    buf = ctypes.create_string_buffer(1 << 12)
    rc = lib().elevate_default_strategy(M, N, K, buf, len(buf))
    if rc != 0:
        raise ValueError(f"elevate_default_strategy: code {rc}")
    return buf.value.decode()


def elevate_dispatch_stats():
    """(applied, failed): how often the dispatch planned a launch from a lowered nest, and how often that failed."""
    a, f = ctypes.c_int64(0), ctypes.c_int64(0)
    lib().elevate_dispatch_stats(ctypes.byref(a), ctypes.byref(f))
    return int(a.value), int(f.value)


def gemm_f32_scheduled(sched: Schedule, A, B, C, transB: bool = False) -> None:
    """C[:] = A @ op(B) with the kernel shape and K split of a schedule."""
    A = _dev_f32(A, "A", 2)
    B = _dev_f32(B, "B", 2)
    C = _dev_f32(C, "C", 2)
    M, K = A.shape
    N = B.shape[0] if transB else B.shape[1]
    if (B.shape[1] if transB else B.shape[0]) != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    _use_current_stream(C)
    _check(lib().gemm_f32_scheduled(ctypes.byref(sched), M, N, K, A.data_ptr(), _ld(A), B.data_ptr(), _ld(B),
                                    C.data_ptr(), _ld(C), int(bool(transB))))
