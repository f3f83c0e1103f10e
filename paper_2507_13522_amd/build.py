"""Compile the HIP library for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "shadow.hip")
DEPS = [SRC, os.path.join(HERE, "csrc", "shadow_kernels.hip.h"),
        os.path.join(os.path.dirname(HERE), "include", "shadow.h")]
LIB = os.path.join(HERE, "libshadow.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                                # every float op rounds on its own
    "-fhip-fp32-correctly-rounded-divide-sqrt",         # IEEE divide and sqrt in float
    "-fno-gpu-flush-denormals-to-zero",                 # keep float denormals
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(d) > t for d in DEPS)


def build_library(force: bool = True, extra_flags=(), out: str = LIB) -> str:
    if not force and not stale():
        return out
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = out + f".tmp{os.getpid()}"
    cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-o", tmp, SRC]
    subprocess.check_call(cmd)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build_library())
