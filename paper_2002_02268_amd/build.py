"""Builds the HIP library in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libgemmf32.so")
OBJ = os.path.join(_HERE, "_build")
# measurement build: the same sources with -DGEMMF32_TIMELINE (per-workgroup timestamps), loaded by bench.py --timeline only
TIMELINE_LIB = os.path.join(_HERE, "libgemmf32_timeline.so")
TIMELINE_OBJ = os.path.join(_HERE, "_build_timeline")
# device code; the kernels of the product are spread over one file per operand layout
SOURCES = ["gemm_f32.hip", "gemm_inst_nn.hip", "gemm_inst_nt.hip", "gemm_inst_packed.hip", "gemm_inst_tn.hip",
           "gemm_inst_tt.hip", "ladder.hip", "binomial.hip"]
# host-only code (the strategy layer)
HOST_SOURCES = ["elevate.cpp", "elevate_api.cpp"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 VALU forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]
HOST_FLAGS = ["-O2", "-std=c++17", "-fPIC"]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES + HOST_SOURCES]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    inc = os.path.join(os.path.dirname(_HERE), "include")
    deps += [os.path.join(inc, f) for f in os.listdir(inc)]
    return any(os.path.getmtime(d) > t for d in deps)


def build_timeline() -> str:
    """Compile the measurement build (libgemmf32_timeline.so)."""
    return build(force=True, extra_flags=("-DGEMMF32_TIMELINE",), lib=TIMELINE_LIB, obj_dir=TIMELINE_OBJ)


def build(force: bool = True, extra_flags=(), lib: str = LIB, obj_dir: str = OBJ) -> str:
    """Compile csrc/ into libgemmf32.so.  Raises CalledProcessError on failure."""
    if force or stale():
        from concurrent.futures import ThreadPoolExecutor
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        os.makedirs(obj_dir, exist_ok=True)

        def compile_one(name):
            obj = os.path.join(obj_dir, name + ".o")
            flags = HOST_FLAGS if name in HOST_SOURCES else [*HIPCC_FLAGS, *extra_flags]
            subprocess.run([hipcc, *flags, "-c", os.path.join(CSRC, name), "-o", obj], check=True)
            return obj

        workers = max(1, min(8, os.cpu_count() or 1))
        with ThreadPoolExecutor(workers) as pool:
            objs = list(pool.map(compile_one, SOURCES + HOST_SOURCES))
        subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs], check=True)
    return lib
