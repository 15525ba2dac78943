"""Phase times of the register-fed convolution kernel on the benchmark's layers.

    python -m paper_2111_00655_amd.phase_probe [--out FILE]

Builds csrc/rf_phase_probe.hip together with csrc/gemm_rf.hip under
-DCLG_RF_STAMPS (the kernels then stamp the device clock at five points; the
library itself is built without the macro) and runs it on 1x1 and 3x3 layers
of ResNet-50 v1.5 at batch 1, each with the K-wave counts the placement search
chooses between.  Needs a GPU.  A developer tool: nothing in the library, the
tests or bench.py depends on it.
"""
from __future__ import annotations

import os
import subprocess
import sys

from . import build as lib_build

PROBE = os.path.join(lib_build.BUILD, "rf_phase_probe")

# tile, images, Cin, Cout, H, filter, stride, pad, waves (0: one chunk per wave; -w: at most w), residual
LAYERS = [
    (16, 1, 1024, 256, 14, 1, 1, 0, 0, 0),     # conv_rf_kernel<16, 1, 16, ...>: sixteen K-waves, one chunk each
    (16, 1, 1024, 256, 14, 1, 1, 0, -4, 0),    # the same layer, four K-waves with four chunks each in flight
    (32, 1, 256, 1024, 14, 1, 1, 0, 0, 1),     # conv_rf_kernel<32, 1, 8, ...>
    (32, 1, 256, 1024, 14, 1, 1, 0, -4, 1),
    (32, 1, 256, 64, 56, 1, 1, 0, 0, 0),
    (16, 1, 64, 256, 56, 1, 1, 0, 0, 1),       # one wave per workgroup
    (16, 1, 2048, 512, 7, 1, 1, 0, 0, 0),
    (16, 1, 2048, 512, 7, 1, 1, 0, -4, 0),
    (32, 1, 64, 64, 56, 3, 1, 1, 0, 0),        # 3x3
    (16, 1, 256, 256, 14, 3, 1, 1, 0, 0),
    (16, 1, 512, 512, 7, 3, 1, 1, 0, 0),
    (32, 1, 3, 64, 224, 7, 2, 3, 0, 0),        # the stem (any-filter path)
]


def build_probe(force: bool = False) -> str:
    src = [os.path.join(lib_build.CSRC, "rf_phase_probe.hip"), os.path.join(lib_build.CSRC, "gemm_rf.hip")]
    os.makedirs(lib_build.BUILD, exist_ok=True)
    newest = max([os.path.getmtime(s) for s in src] + [lib_build._headers_mtime()])
    if not force and os.path.exists(PROBE) and os.path.getmtime(PROBE) >= newest:
        return PROBE
    cmd = [lib_build.HIPCC, "-O3", "-std=c++17", "-DCLG_RF_STAMPS", "-I", lib_build.INCLUDE, "-I", lib_build.CSRC] + lib_build.DEVICE
    cmd += ["-o", PROBE] + src
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on the phase probe:\n" + "\n".join(
            l for l in (r.stdout + r.stderr).splitlines() if "packed-fp32-ops" not in l))
    return PROBE


def main():
    out = sys.stdout
    if "--out" in sys.argv:
        path = sys.argv[sys.argv.index("--out") + 1]
        os.makedirs(os.path.dirname(os.path.abspath(path)), exist_ok=True)
        out = open(path, "w")
    probe = build_probe()
    rc = 0
    for layer in LAYERS:
        r = subprocess.run([probe] + [str(v) for v in layer], capture_output=True, text=True, timeout=120)
        out.write(r.stdout)
        out.flush()
        if r.returncode != 0:
            out.write(f"(probe exited with status {r.returncode}) {r.stderr}\n")
            rc = 1
            break                          # nothing more is started after a failure
    return rc


if __name__ == "__main__":
    sys.exit(main())
