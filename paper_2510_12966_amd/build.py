"""Builds libpsd.so (the HIP library, gfx950) in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpsd.so")
SYNTH_DEV_SRC = os.path.join(HERE, "synth", "synth_dev.hip")
SYNTH_DEV_LIB = os.path.join(HERE, "synth", "libsynth_dev.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # no packed-fp32 instruction selection (some forms have been unreliable on these machines)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _hipcc(cmd, verbose):
    res = subprocess.run(cmd, capture_output=True, text=True)
    log = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log, file=sys.stderr)


def build(verbose: bool = False) -> str:
    """Compiles every HIP source into libpsd.so, and the device-side input generator of the acceptance microbenchmark
    into synth/libsynth_dev.so; always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    _hipcc([hipcc] + HIPCC_FLAGS + ["-I", os.path.join(os.path.dirname(HERE), "include"), "-o", LIB] + sources(), verbose)
    _hipcc([hipcc] + HIPCC_FLAGS + ["-o", SYNTH_DEV_LIB, SYNTH_DEV_SRC], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
