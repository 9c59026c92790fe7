"""Builds libtp_pack.so (host C++ + HIP kernels for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(os.path.dirname(PKG_DIR), "include")
LIB_PATH = os.path.join(PKG_DIR, "libtp_pack.so")

SOURCES = ["api.cpp", "static_staging.cpp", "model_api.cpp", "model.cpp", "resource_api.cpp", "resource_cache.cpp", "type_tree.cpp",
           "canon.cpp", "plan.cpp", "kernels.hip"]


def hipcc() -> str:
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build(verbose: bool = False) -> str:
    """Compile every source for gfx950 and link the shared library.  Always recompiles."""
    cmd = [
        hipcc(), "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
        # this pool: never let the compiler form packed-fp32 instructions
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
        "-I", INCLUDE, "-I", CSRC,
    ]
    for s in SOURCES:
        if s.endswith(".cpp"):
            cmd += ["-x", "hip", os.path.join(CSRC, s)]
        else:
            cmd += [os.path.join(CSRC, s)]
    cmd += ["-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    for tool in C_TOOLS:
        build_c_tool(tool)
    return LIB_PATH


# plain-C programs that use the library through include/tp_pack.h alone
C_TOOLS = ("commit_timing", "resource_timing", "pack_selftest")
TIMING_EXE = os.path.join(PKG_DIR, "commit_timing")
RESOURCE_TIMING_EXE = os.path.join(PKG_DIR, "resource_timing")
SELFTEST_EXE = os.path.join(PKG_DIR, "pack_selftest")


def build_c_tool(name: str) -> str:
    """Compiles csrc/<name>.c with gcc and links it against the library just built."""
    exe = os.path.join(PKG_DIR, name)
    subprocess.check_call([
        "gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-I", INCLUDE, os.path.join(CSRC, name + ".c"),
        "-L", PKG_DIR, "-ltp_pack", "-Wl,-rpath,$ORIGIN", "-Wl,-rpath-link," + "/opt/rocm/lib", "-o", exe,
    ])
    return exe


if __name__ == "__main__":
    build(verbose=True)
    print(LIB_PATH)
    sys.exit(0)
