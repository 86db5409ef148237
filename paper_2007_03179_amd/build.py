"""Build the HIP library (hipcc, gfx950) in-tree as paper_2007_03179_amd/libgespmm.so."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "gespmm.hip")
LIB = os.path.join(HERE, "libgespmm.so")

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    "-munsafe-fp-atomics",                                   # hardware fp32 atomic add
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"),
]


def build(force: bool = True, extra=()) -> str:
    """Compile csrc/gespmm.hip.  force=False reuses an existing library."""
    if not force and os.path.exists(LIB):
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.run([hipcc, *HIPCC_FLAGS, *extra, "-o", LIB, SRC], check=True)
    return LIB


CUSTOM_SRC = os.path.join(ROOT, "tests", "custom_ops", "custom_ops.hip")
CUSTOM_LIB = os.path.join(ROOT, "tests", "custom_ops", "libcustom_ops.so")


def build_custom_example(force: bool = True) -> str:
    """Compile the two example user-defined reduce operations (tests/custom_ops)."""
    if not force and os.path.exists(CUSTOM_LIB):
        return CUSTOM_LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.run([hipcc, *HIPCC_FLAGS, "-o", CUSTOM_LIB, CUSTOM_SRC], check=True)
    return CUSTOM_LIB


if __name__ == "__main__":
    print(build())
    print(build_custom_example())
