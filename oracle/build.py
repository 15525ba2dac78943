"""Compile the oracle's C operators (ops.c) into liboracle_ops.so with gcc.

Test infrastructure only: building the checker is not using it.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ops.c")
LIB = os.path.join(HERE, "liboracle_ops.so")


LIB_SAN = os.path.join(HERE, "liboracle_ops_san.so")
CLANG = os.environ.get("ORACLE_CLANG", "/opt/rocm/lib/llvm/bin/clang")


def build(force: bool = False) -> str:
    # ORACLE_OPS_LIBRARY selects a library built elsewhere (the sanitized one below)
    if os.environ.get("ORACLE_OPS_LIBRARY"):
        return os.environ["ORACLE_OPS_LIBRARY"]
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= os.path.getmtime(SRC)):
        return LIB
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
           "-ffp-contract=off", "-Wall", "-Wextra", "-o", tmp, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


def build_sanitized() -> str:
    """The same operators with AddressSanitizer + UndefinedBehaviorSanitizer, built with clang so that it
    shares one sanitizer runtime with the sanitized build of the GPU library's host code (the process
    preloads that runtime).  The arithmetic flags are the same, so the results are too."""
    tmp = LIB_SAN + f".tmp{os.getpid()}"
    cmd = [CLANG, "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fsanitize=address", "-fsanitize=undefined", "-fno-omit-frame-pointer", "-shared-libsan",
           "-Wall", "-Wextra", "-o", tmp, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB_SAN)
    return LIB_SAN


if __name__ == "__main__":
    import sys
    print(build_sanitized() if "--sanitize" in sys.argv else build(force=True))
