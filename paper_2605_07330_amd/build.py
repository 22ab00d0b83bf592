"""Builds libsrs.so (HIP, gfx950 only) in-tree, next to this file."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libsrs.so")
SOURCES = [os.path.join(HERE, "csrc", "srs.hip")]
HEADERS = [os.path.join(HERE, "csrc", "srs_kernels.hpp"), os.path.join(ROOT, "include", "srs.h")]


def hipcc_command(out: str = LIB, extra=()) -> list:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wall", "-Wno-unused-command-line-argument",
            "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
            "-Wl,-rpath,/opt/rocm/lib", *extra, *SOURCES, "-o", out]


def build_lib(verbose: bool = False) -> str:
    cmd = hipcc_command()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def build_lib_host_sanitized(out: str, verbose: bool = False) -> str:
    """libsrs.so with its HOST code under AddressSanitizer and UndefinedBehaviorSanitizer (device code as usual),
    for CPU-only runs of the host-side tests (bucket / segment / tile tables, argument checks) with SRS_LIBRARY
    pointing at it and clang's ASan runtime preloaded.  Never meant for a GPU machine."""
    cmd = hipcc_command(out, extra=["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                                    "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-shared-libsan"])
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return out


def clang_asan_runtime() -> str:
    import glob
    hits = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    return hits[-1] if hits else ""


C_CONSUMER_SRC = os.path.join(ROOT, "tests", "c_abi", "roundtrip.c")
C_CONSUMER = os.path.join(ROOT, "tests", "c_abi", "roundtrip")


def build_c_consumer(verbose: bool = False) -> str:
    """The plain C program the GPU tests run against libsrs.so (gcc, C99: the header must be valid C)."""
    gcc = os.environ.get("CC", "gcc")
    cmd = [gcc, "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           "-isystem", "/opt/rocm/include", C_CONSUMER_SRC, "-o", C_CONSUMER,
           "-L", HERE, "-lsrs", "-L", "/opt/rocm/lib", "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../../paper_2605_07330_amd", "-Wl,-rpath,/opt/rocm/lib"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return C_CONSUMER


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


if __name__ == "__main__":
    build_lib(verbose=True)
    build_c_consumer(verbose=True)
    print(LIB)
