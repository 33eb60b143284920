"""The division by a launch constant that the kernels use to turn a workgroup id into tile coordinates
(csrc/fast_div.hpp), checked on the host against the C++ division."""
from __future__ import annotations

import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_fast_division_agrees_with_division(tmp_path):
    exe = tmp_path / "fast_div_check"
    subprocess.run(["g++", "-O2", "-std=c++17", "-I", os.path.join(ROOT, "paper_2002_02268_amd", "csrc"),
                    os.path.join(ROOT, "tests", "fast_div_check.cpp"), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    assert out.startswith("ok "), out
