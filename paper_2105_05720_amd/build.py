"""Builds libccfused.so for gfx950 with hipcc, in-tree (next to this file).

The library is several translation units (one per kernel family) only so that they compile side by side; each is
compiled to an object file and the objects are linked into one shared library, whose dynamic symbol table is cut down
to the C ABI by csrc/exports.map."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
SOURCES = [os.path.join(CSRC, n) for n in ("ccfused.hip", "launch_adam_f16.hip", "launch_adam_f32.hip", "launch_lamb.hip",
                                           "launch_unfused.hip")]
EXPORTS_MAP = os.path.join(CSRC, "exports.map")
DEPS = SOURCES + [os.path.join(CSRC, "kernels.hip.h"), os.path.join(CSRC, "plan.hpp"), os.path.join(CSRC, "launch_adam.inc.hpp"),
                  os.path.join(ROOT, "include", "ccfused.h"), EXPORTS_MAP]
LIB = os.path.join(_HERE, "libccfused.so")
OBJ_DIR = os.path.join(_HERE, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fvisibility=hidden",
    "-ffp-contract=off",                                              # fused multiply-adds are written out by hand
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",      # no packed-fp32 instructions
    # The kernels issue their counting atomics (flag count, chunk ticket) early and look at the result a block of work
    # later.  The compiler's wave-level atomic aggregation would rewrite each into "one lane adds, readfirstlane the
    # result", which needs the result at once and so drains the wave's memory counter right behind the atomic.
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
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
    os.makedirs(OBJ_DIR, exist_ok=True)
    tag = ".%d" % os.getpid()
    objs = [os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + tag + ".o") for src in SOURCES]

    def compile_one(pair):
        src, obj = pair
        subprocess.check_call([HIPCC] + FLAGS + list(extra) + ["-c", "-o", obj, src])
    try:
        with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
            list(pool.map(compile_one, zip(SOURCES, objs)))
        tmp = LIB + ".tmp%d" % os.getpid()
        subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-Wl,--version-script=" + EXPORTS_MAP,
                               "-o", tmp] + objs)
        os.replace(tmp, LIB)
    finally:
        for obj in objs:
            if os.path.exists(obj):
                os.remove(obj)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True, extra=sys.argv[1:]))
