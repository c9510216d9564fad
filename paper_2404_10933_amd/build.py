"""Builds libllmem.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libllmem.so")
SOURCES = ("estimate.hip", "estimate_batch.hip", "decide.hip", "timeline.hip", "generate.hip")
HIPCC_FLAGS = ("--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops")


def build(verbose: bool = False) -> str:
    """Compile every HIP source into the shared library; always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        hipcc = "hipcc"
    cmd = [hipcc, *HIPCC_FLAGS, "-o", LIB, *(os.path.join(CSRC, s) for s in SOURCES)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose:
        print(res.stderr)
    return LIB


def build_calibrate() -> str:
    """Compile the stand-alone calibration program (instruction issue rates, HBM read rate)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        hipcc = "hipcc"
    exe = os.path.join(HERE, "calibrate")
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-O2", "-Xclang", "-target-feature", "-Xclang",
                          "-packed-fp32-ops", "-o", exe, os.path.join(CSRC, "calibrate.hip")],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return exe


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_calibrate())
