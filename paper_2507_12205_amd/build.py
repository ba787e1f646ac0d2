"""Builds libecspmv.so (host encoder + HIP kernels for gfx950 + C ABI) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libecspmv.so")
TRACE_LIB = os.path.join(PKG, "libecspmv_trace.so")     # the same sources with clock stamps compiled in (timeline.py)
SOURCES = ["api.cpp", "encoder.cpp", "kernels.hip"]
HEADERS = ["encoder.h", "launch.h", "ecspmv_format.h", os.path.join("..", "..", "include", "ecspmv.h")]


def lib_path() -> str:
    """Path of the shared library; ECSPMV_LIB overrides it (to try a differently built library)."""
    return os.environ.get("ECSPMV_LIB", LIB)


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build_all(verbose: bool = False) -> None:
    """The product library and the stamped one for the timeline script."""
    build(verbose)
    build(verbose, extra_flags=("-DECS_TRACE=1",), out=TRACE_LIB)


def build(verbose: bool = False, extra_flags=(), out: str = LIB) -> str:
    """Compile every source for gfx950 and link the shared library.  Needs hipcc; no GPU required."""
    cmd = ["hipcc", "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           # the first kernel arguments (count, workgroup size, first item of a launch) arrive in registers
           "-mllvm", "-amdgpu-kernarg-preload-count=16",
           "-mpopcnt", "-pthread", "-Wall", "-Wno-unused-function",
           "-x", "hip"]
    cmd += list(extra_flags)
    cmd += [os.path.join(CSRC, f) for f in SOURCES]
    cmd += ["-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr[-4000:])
    return out


if __name__ == "__main__":
    print(build(verbose=True))
