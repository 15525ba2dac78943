#!/usr/bin/env python3
"""Runs the CPU test suite (-m "not gpu") with AddressSanitizer and UndefinedBehaviorSanitizer on the
host code of the GPU library (graph, matcher, search, lowering, workspace planner, C ABI) and on the
oracle's C operators.

    python tests/run_sanitized.py [pytest arguments]

Builds paper_2111_00655_amd/libcollage_mi_san.so and oracle/liboracle_ops_san.so, then starts pytest in
a child process that preloads the sanitizer runtime and loads those two libraries instead of the normal
ones.  Any report ends the run with a non-zero status.  No GPU is involved: contexts are host-only.
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    from paper_2111_00655_amd import build as lib_build
    from oracle import build as oracle_build
    lib = lib_build.build(sanitize=True)
    ops = oracle_build.build_sanitized()
    env = dict(os.environ)
    pre = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = lib_build.san_runtime() + (":" + pre if pre else "")
    env["CLG_LIBRARY"] = lib
    env["ORACLE_OPS_LIBRARY"] = ops
    # Python itself leaks at exit by design; everything else stops at the first report
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    args = sys.argv[1:] or ["tests", "-x", "-q", "-m", "not gpu"]
    return subprocess.call([sys.executable, "-m", "pytest"] + args, cwd=ROOT, env=env)


if __name__ == "__main__":
    sys.exit(main())
