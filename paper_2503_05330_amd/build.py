"""Compiles the HIP sources under csrc/ into libcsd.so (gfx950 only)."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = [os.path.join(HERE, "csrc", "csd.hip")]
LIBRARY = os.path.join(HERE, "libcsd.so")

# -packed-fp32-ops is switched off on purpose: the compiler must not form packed
# FP32 instructions from ordinary float code in this library.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_library() -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        raise RuntimeError("hipcc not found: the csd HIP library cannot be built")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-o", LIBRARY, *SOURCES]
    subprocess.check_call(cmd)
    return LIBRARY


if __name__ == "__main__":
    print(build_library())
