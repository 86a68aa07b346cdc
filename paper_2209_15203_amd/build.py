"""Compile libbts.so (hand-written HIP for gfx950) and the measurement instrument
libbts_probe.so in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libbts.so")
PROBE_LIB = os.path.join(HERE, "libbts_probe.so")
PROBE_SRC = os.path.join(CSRC, "probe.hip")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                 # the only fusions are the explicit __fmaf_rn calls
    "-fno-fast-math", "-fno-gpu-flush-denormals-to-zero",   # keep fp32 denormals
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


# The packed-fp32 feature switch is meant for the device pass.  hipcc hands -Xclang options
# to the host pass too (-Xarch_device cannot forward an option that takes an argument), and
# the host pass answers with this line once per file; it is dropped from the output.
_HOST_NOISE = "'-packed-fp32-ops' is not a recognized feature for this target"


def sources():
    """Sources of libbts.so: every .hip file but the probe's."""
    return sorted(f for f in glob.glob(os.path.join(CSRC, "*.hip")) if f != PROBE_SRC)


def _compile(out: str, srcs, verbose: bool) -> None:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-o", out] + list(srcs)
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if _HOST_NOISE not in l)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + err + "\n")
        raise RuntimeError("hipcc failed")
    if verbose and err.strip():
        sys.stderr.write(err + "\n")


def build(verbose: bool = False) -> str:
    _compile(LIB, sources(), verbose)
    _compile(PROBE_LIB, [PROBE_SRC], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
