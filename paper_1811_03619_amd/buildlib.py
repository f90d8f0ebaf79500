"""Builds ``libpipesgd.so`` (HIP kernels + C ABI) for gfx950 with hipcc.

hipcc cross-compiles without a GPU.  The library is placed inside the package
so that it travels with the source tree.
"""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB_PATH = os.path.join(_HERE, "libpipesgd.so")

SOURCES = ["pipesgd_kernels.hip", "pipesgd_runtime.hip", "pipesgd_host.cpp"]
HEADERS = ["pipesgd_device.hpp", "pipesgd_internal.hpp"]      # private to csrc/

# One IEEE rounding per written operation: no contraction, no fast-math.
# Packed-fp32 instruction selection is switched off on purpose.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    deps = sources() + [os.path.join(CSRC, h) for h in HEADERS] + [os.path.join(INCLUDE, "pipesgd.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False, defines=(), out: str = LIB_PATH) -> str:
    """Compile the library.  force=False skips the work if the library is newer
    than its sources.  `defines` ("NAME=VALUE") and `out` build a tuning variant
    somewhere else."""
    if not force and out == LIB_PATH and not is_stale():
        return LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", INCLUDE] + ["-D" + d for d in defines]
    for s in sources():
        cmd += ["-x", "hip", s]
    cmd += ["-o", out]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return out


if __name__ == "__main__":
    print(build(force=True, verbose=True))
