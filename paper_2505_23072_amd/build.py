"""Builds libfst.so (host parser/planner/stager + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfst.so")
SOURCES = ["header.cpp", "plan.cpp", "kernels.hip", "materialize.hip", "static_ws.hip", "stage.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def sources_newer_than_lib() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "fst.h")]
    return any(os.path.getmtime(d) > t for d in deps)


# Flags that decide the generated gfx950 code (the assembly guard in the tests compiles with the same).
DEVICE_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17",
                # packed fp32 instructions stay off
                "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(verbose: bool = False) -> str:
    cmd = [HIPCC] + DEVICE_FLAGS + ["-fPIC", "-shared", "-pthread", "-Wall", "-Wextra", "-Wno-unused-parameter",
                                    "-o", LIB]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    print(LIB)
