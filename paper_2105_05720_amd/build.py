"""Builds libccfused.so for gfx950 with hipcc, in-tree (next to this file)."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
SRC = os.path.join(_HERE, "csrc", "ccfused.hip")
DEPS = [SRC, os.path.join(_HERE, "csrc", "kernels.hip.h"), os.path.join(ROOT, "include", "ccfused.h")]
LIB = os.path.join(_HERE, "libccfused.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-ffp-contract=off",                                              # fused multiply-adds are written out by hand
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",      # no packed-fp32 instructions
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(_HERE, "csrc"),
]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(d) > t for d in DEPS)


def build_library(force: bool = True, extra=()) -> str:
    """Compile the HIP library.  force=False skips the compile when the built file is newer than its sources."""
    if not force and not is_stale():
        return LIB
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [HIPCC] + FLAGS + list(extra) + ["-o", tmp, SRC]
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True, extra=sys.argv[1:]))
