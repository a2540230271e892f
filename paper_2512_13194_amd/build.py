"""Builds the HIP library (libears.so) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libears.so")
SOURCES = [os.path.join(CSRC, "ears_kernels.hip")]
HEADERS = [os.path.join(CSRC, h) for h in ("ears_device.h", "row_stats.h", "decide.h", "sample.h",
                                            "verify.h", "greedy.h", "lm_head.h", "bench_aids.h")]
HEADERS.append(os.path.join(os.path.dirname(_HERE), "include", "ears.h"))

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # no implicit mul+add fusion: the kernels rely on fl(m*c) being the rounded product and
    # write fmaf() where a fused operation is wanted
    "-ffp-contract=off",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def build(verbose: bool = False, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + ["-o", tmp] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=sys.argv[1:]))
