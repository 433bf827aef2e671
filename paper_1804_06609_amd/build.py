"""Builds libdba.so (HIP, gfx950 only) next to this file."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdba.so")
SOURCES = [os.path.join(CSRC, "dba.hip")]
DEPS = SOURCES + [os.path.join(CSRC, f) for f in ("dba_kernels.hpp", "wave_topk.hpp")] + [
    os.path.join(os.path.dirname(HERE), "include", f) for f in ("dba.h", "dba_debug.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC", "-fvisibility=hidden",
    # packed fp32 VALU forms are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    # leading scalar kernel arguments arrive in registers at wave start (no load, no wait)
    "-mllvm", "-amdgpu-kernarg-preload-count=8",
]


def build(force: bool = True, extra=()) -> str:
    stale = force or not os.path.exists(LIB) or any(
        os.path.getmtime(LIB) < os.path.getmtime(d) for d in DEPS)
    if stale:
        cmd = [HIPCC] + FLAGS + list(extra) + SOURCES + ["-o", LIB]
        subprocess.check_call(cmd)
    return LIB


EXAMPLE_SRC = os.path.join(os.path.dirname(HERE), "examples", "decode_from_file.c")
EXAMPLE_BIN = os.path.join(os.path.dirname(HERE), "examples", "decode_from_file")


def build_example() -> str:
    """Compiles the plain-C caller of the library with the host C compiler (no hipcc: the
    boundary is a C ABI) and links it against libdba.so and the HIP runtime."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    subprocess.check_call([
        "gcc", "-O1", "-Wall", "-std=c11", "-D__HIP_PLATFORM_AMD__", f"-I{rocm}/include", EXAMPLE_SRC,
        "-o", EXAMPLE_BIN, f"-L{rocm}/lib", "-lamdhip64", f"-L{HERE}", "-ldba",
        "-Wl,-rpath,$ORIGIN/../paper_1804_06609_amd", f"-Wl,-rpath,{rocm}/lib"])
    return EXAMPLE_BIN


if __name__ == "__main__":
    print(build(force=True, extra=sys.argv[1:]))
    print(build_example())
