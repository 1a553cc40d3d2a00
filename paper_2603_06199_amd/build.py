"""Builds the gfx950 shared library in-tree with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libflashprefill.so")
PROBE = os.path.join(HERE, "mfma_probe")     # stand-alone measurement aid (bench.py --mfma-probe), not part of the library
SOURCES = ["flashprefill.hip"]
HEADERS = ["fp_device.hpp", "fp_search.hpp", "fp_attn.hpp"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instruction selection is switched off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # device code only: NaNs are not honoured (infinities still are; the kernels use -inf as the
    # masked-logit value), which lets max reductions compile to v_max3_f32 without canonicalising
    "-Xarch_device", "-fno-honor-nans",
    "-Wall", "-Wno-unused-function",
]


# The kernels carry inline assembly whose correctness leans on this compiler's register handling
# (loads issued from assembly whose results are first touched behind an explicit s_waitcnt, a
# hand-placed s_nop before v_permlane32_swap): the GPU tests were run with this toolchain, and a
# different one has to pass them again before its output is trusted.
TESTED_HIPCC = "7.2"


def hipcc_version(hipcc: str) -> str:
    try:
        out = subprocess.run([hipcc, "--version"], capture_output=True, text=True).stdout
        for line in out.splitlines():
            if line.startswith("HIP version:"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.join(HERE, "..", "include", "flashprefill.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if force or stale():
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        ver = hipcc_version(hipcc)
        if not ver.startswith(TESTED_HIPCC):
            print(f"warning: hipcc {ver} is not the tested {TESTED_HIPCC}.x: run the GPU tests before relying on this build",
                  file=sys.stderr, flush=True)
        cmd = [hipcc] + HIPCC_FLAGS + ["-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        probe = [hipcc] + [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")] + ["-o", PROBE, os.path.join(CSRC, "mfma_probe.hip")]
        if verbose:
            print(" ".join(probe), flush=True)
        subprocess.run(probe, check=True)
    return LIB


if __name__ == "__main__":
    build(force=True, verbose=True)
    print(LIB)
