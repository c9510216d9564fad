"""Builds libllmem.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libllmem.so")
SOURCES = ("estimate.hip", "estimate_batch.hip", "specialize.hip", "decide.hip", "timeline.hip", "generate.hip")
# what the run-time build of the specialized kernel compiles: the kernel source first, then the
# headers it includes, each under its bare name
EMBEDDED = (("estimate_batch.hip", os.path.join(CSRC, "estimate_batch.hip")),
            ("llmem.h", os.path.join(HERE, "..", "include", "llmem.h")),
            ("estimate_args.h", os.path.join(CSRC, "estimate_args.h")),
            ("grid_draws.h", os.path.join(CSRC, "grid_draws.h")),
            ("wave.h", os.path.join(CSRC, "wave.h")))
HIPCC_FLAGS = ("--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops")


def write_embedded_sources() -> str:
    """csrc/embedded_sources.inc: the kernel source and its headers as string literals."""
    out = ["// written by build.py from the files next to it; not edited by hand",
           f"static const int EMBEDDED_COUNT = {len(EMBEDDED)};",
           "static const char *const EMBEDDED_NAMES[] = {" + ", ".join(f'"{n}"' for n, _ in EMBEDDED) + "};",
           "static const char *const EMBEDDED_TEXTS[] = {"]
    for _, path in EMBEDDED:
        text = open(path).read()
        assert ')LLMEM_SRC"' not in text
        # string literals are limited in length by some compilers: one literal per 8 KB, concatenated
        chunks = [text[i:i + 8192] for i in range(0, len(text), 8192)]
        out.append("\n".join(f'R"LLMEM_SRC({c})LLMEM_SRC"' for c in chunks) + ",")
    out.append("};")
    path = os.path.join(CSRC, "embedded_sources.inc")
    with open(path, "w") as f:
        f.write("\n".join(out) + "\n")
    return path


def build(verbose: bool = False) -> str:
    """Compile every HIP source into the shared library; always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        hipcc = "hipcc"
    write_embedded_sources()
    cmd = [hipcc, *HIPCC_FLAGS, "-o", LIB, *(os.path.join(CSRC, s) for s in SOURCES), "-lhiprtc"]
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
