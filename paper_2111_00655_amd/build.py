"""Builds libcollage_mi.so (host C++ and gfx950 HIP kernels) in-tree with hipcc.

    python -m paper_2111_00655_amd.build [--force] [--sanitize]

Objects go to paper_2111_00655_amd/_build/, the library next to this file.
A source is recompiled when it, or any header, is newer than its object.

--sanitize builds a second library, libcollage_mi_san.so (objects in
_build_san/), whose HOST code is instrumented with AddressSanitizer and
UndefinedBehaviorSanitizer (the device code is compiled as usual: GPU
sanitizers are not used).  It is for CPU-only runs of the host logic - graph,
matcher, search, lowering, workspace planning - in host-only contexts: set
CLG_LIBRARY to its path and preload the sanitizer runtime (SAN_RUNTIME below)
before starting Python.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libcollage_mi.so")

SOURCES = ["graph.cpp", "matcher.cpp", "search.cpp", "lower.cpp", "plan.cpp",
           "profiler.cpp", "rules.cpp", "evolve.cpp", "capi.cpp", "kernels_gemm.hip", "gemm_fast_mm.hip", "gemm_fast_conv.hip",
           "gemm_lean_mm.hip", "gemm_lean_conv.hip", "gemm_rf.hip",
           "kernels_misc.hip", "sepconv.hip", "attention.hip", "static_ws.hip"]

BUILD_SAN = os.path.join(HERE, "_build_san")
LIB_SAN = os.path.join(HERE, "libcollage_mi_san.so")
SAN_FLAGS = ["-fsanitize=address", "-fsanitize=undefined"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra", "-Wno-unused-parameter",
          "-I", INCLUDE, "-I", CSRC]
# no packed-fp32 instructions: plain v_fma_f32 / v_add_f32 only
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _headers_mtime() -> float:
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs += [os.path.join(INCLUDE, f) for f in os.listdir(INCLUDE) if f.endswith(".h")]
    return max(os.path.getmtime(h) for h in hs)


def san_runtime() -> str:
    """Path of the shared AddressSanitizer runtime of hipcc's clang (to be preloaded into Python)."""
    r = subprocess.run([HIPCC, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    return os.path.realpath(r.stdout.strip())


def _compile(src: str, force: bool, hdr_mtime: float, sanitize: bool = False) -> str:
    path = os.path.join(CSRC, src)
    obj = os.path.join(BUILD_SAN if sanitize else BUILD, src + ".o")
    if (not force and os.path.exists(obj)
            and os.path.getmtime(obj) >= max(os.path.getmtime(path), hdr_mtime)):
        return obj
    cmd = [HIPCC] + COMMON
    if src.endswith(".hip"):
        cmd += DEVICE
        if sanitize:                         # host pass only: each flag directly behind -Xarch_host
            for f in SAN_FLAGS:
                cmd += ["-Xarch_host", f]
            cmd += ["-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    else:
        cmd += ["-x", "c++", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include"]
        if sanitize:
            cmd += SAN_FLAGS + ["-fno-omit-frame-pointer", "-g"]
    cmd += ["-c", path, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                     if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{msgs}")
    if msgs.strip():
        print(msgs, file=sys.stderr)
    return obj


def build(force: bool = False, verbose: bool = False, sanitize: bool = False) -> str:
    lib = LIB_SAN if sanitize else LIB
    os.makedirs(BUILD_SAN if sanitize else BUILD, exist_ok=True)
    hdr = _headers_mtime()
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(lambda s: _compile(s, force, hdr, sanitize), SOURCES))
    if (force or not os.path.exists(lib)
            or os.path.getmtime(lib) < max(os.path.getmtime(o) for o in objs)):
        tmp = lib + f".tmp{os.getpid()}"
        cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs
        if sanitize:                         # the runtime stays a shared library that the process preloads
            cmd += SAN_FLAGS + ["-shared-libsan", "-fno-gpu-sanitize"]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
        os.replace(tmp, lib)
    if verbose:
        print(lib)
        if sanitize:
            print("SAN_RUNTIME=" + san_runtime())
    return lib


if __name__ == "__main__":
    build(force="--force" in sys.argv, verbose=True, sanitize="--sanitize" in sys.argv)
