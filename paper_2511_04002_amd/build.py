"""Builds libtsq.so (the C-ABI library) for gfx950 with hipcc, in-tree.

Usage: python -m paper_2511_04002_amd.build [--force]
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtsq.so")
SOURCES = ["tsq_api.hip", "tsq_kernels.hip", "tsq_fused.hip", "tsq_entropy.hip", "tsq_rans.hip", "tsq_link.cpp"]
HEADERS = ["tsq_internal.hpp", "tsq_device.hpp", os.path.join(ROOT, "include", "tsq.h")]

# -ffp-contract=off: the quantizer's multiply and every fp64 product of the budget test must
#   stay single IEEE operations; -packed-fp32-ops off: scalar fp32 code is not merged into
#   packed fp32 instructions.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    return "hipcc"


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + [h if os.path.isabs(h) else os.path.join(CSRC, h) for h in HEADERS]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, extra=()) -> str:
    if force or stale():
        tmp = LIB + ".tmp.%d" % os.getpid()
        cmd = [hipcc()] + FLAGS + list(extra) + ["-o", tmp] + [os.path.join(CSRC, s) for s in SOURCES]
        subprocess.run(cmd, check=True)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
