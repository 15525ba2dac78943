"""Cost of a layer boundary inside one persistent kernel against a kernel launch.

    python -m paper_2111_00655_amd.barrier_probe [--out FILE]

Builds and runs csrc/grid_barrier_probe.hip (see its header).  Needs a GPU.  A
developer tool behind a design decision (the library runs one kernel per fused
group and fuses sibling kernels, not chains): nothing else depends on it.
"""
from __future__ import annotations

import os
import subprocess
import sys

from . import build as lib_build

PROBE = os.path.join(lib_build.BUILD, "grid_barrier_probe")


def build_probe(force: bool = False) -> str:
    src = os.path.join(lib_build.CSRC, "grid_barrier_probe.hip")
    os.makedirs(lib_build.BUILD, exist_ok=True)
    if not force and os.path.exists(PROBE) and os.path.getmtime(PROBE) >= os.path.getmtime(src):
        return PROBE
    cmd = [lib_build.HIPCC, "-O3", "-std=c++17"] + lib_build.DEVICE + ["-o", PROBE, src]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on the barrier probe:\n" + "\n".join(
            l for l in (r.stdout + r.stderr).splitlines() if "packed-fp32-ops" not in l))
    return PROBE


def main():
    r = subprocess.run([build_probe()], capture_output=True, text=True, timeout=120)
    if "--out" in sys.argv:
        path = sys.argv[sys.argv.index("--out") + 1]
        os.makedirs(os.path.dirname(os.path.abspath(path)), exist_ok=True)
        with open(path, "w") as f:
            f.write(r.stdout)
    sys.stdout.write(r.stdout)
    sys.stderr.write(r.stderr)
    return r.returncode


if __name__ == "__main__":
    sys.exit(main())
