"""Build libstq.so (the C-ABI library) for gfx950 with hipcc, in-tree next to the sources."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libstq.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -ffp-contract=off: every fp32 operation of the step is rounded on its own (the packed codes
# must be reproducible bit for bit).  Packed-fp32 instructions are disabled.
DEVICE_FLAGS = ["--offload-arch=gfx950", "-ffp-contract=off",
                "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
COMMON = ["-O3", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
          "-Wall", "-Wextra", "-Wno-unused-parameter"]

SOURCES = ["stq_step.hip", "stq_kernels.hip", "stq_engine.hip", "stq_api.cpp", "stq_tables.cpp", "stq_decide.cpp"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    cmd = [HIPCC, *COMMON]
    if src.endswith(".hip") or src == "stq_api.cpp":
        cmd += ["-x", "hip", *DEVICE_FLAGS]
    else:
        cmd += ["-ffp-contract=off"]
    cmd += ["-c", path, "-o", obj]
    subprocess.check_call(cmd)
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", tmp])
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
