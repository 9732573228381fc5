"""Builds libsparbit.so (HIP kernels + C-ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libsparbit.so")
ARCH = "gfx950"
SOURCES = ["api.hip", "plan.cpp"]
HEADERS = ["kernels.hip.hpp", "plan.hpp", os.path.join("..", "..", "include", "sparbit.h")]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the HIP library cannot be built")
    return exe


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build_library(force: bool = False, verbose: bool = False) -> str:
    """Compile every HIP/C++ source into one shared library for gfx950."""
    if not force and not is_stale():
        return LIB_PATH
    tmp = LIB_PATH + f".tmp{os.getpid()}"
    objdir = os.path.join(_HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    api_o, plan_o = os.path.join(objdir, "api.o"), os.path.join(objdir, "plan.o")
    # One source per hipcc call: with several inputs of mixed language on one
    # line the wrapper drops --offload-arch and falls back to its default target.
    cmds = [
        [_hipcc(), "-O3", "-std=c++17", f"--offload-arch={ARCH}", "-fPIC", "-Wall",
         # no packed-fp32 instruction forms in any device code of this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-c", os.path.join(CSRC, "api.hip"), "-o", api_o],
        ["g++", "-O2", "-std=c++17", "-fPIC", "-Wall", "-c", os.path.join(CSRC, "plan.cpp"), "-o", plan_o],
        [_hipcc(), f"--offload-arch={ARCH}", "-shared", "-fPIC", api_o, plan_o, "-o", tmp],
    ]
    for cmd in cmds:
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("build failed: " + " ".join(cmd) + "\n" + res.stdout + res.stderr)
        noise = "is not a recognized feature for this target"  # host pass does not know the device feature
        msgs = [l for l in res.stderr.splitlines() if l.strip() and noise not in l]
        if verbose and msgs:
            print("\n".join(msgs))
    with open(tmp, "rb") as fh:
        if f"hipv4-amdgcn-amd-amdhsa--{ARCH}".encode() not in fh.read():
            os.unlink(tmp)
            raise RuntimeError(f"built library carries no {ARCH} code object")
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
