"""Build libgoodroute.so for gfx950 with hipcc (in-tree, next to the sources)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(CSRC, "libgoodroute.so")
SOURCES = ["api.hip", "status.hip", "score.hip"]


def hipcc_command() -> list:
    return ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
            "-ffp-contract=off",
            # packed-FP32 instructions stay off: ordinary float code must not be fused into them
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-I", os.path.join(ROOT, "include"),
            "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]


def build_library(verbose: bool = False) -> str:
    cmd = hipcc_command()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


PROBE = os.path.join(CSRC, "probe_valu_issue")


def build_probe(verbose: bool = False) -> str:
    """The stand-alone microbenchmark behind the vector-ALU issue model (not part of the library)."""
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-o", PROBE, PROBE + ".hip"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return PROBE


if __name__ == "__main__":
    build_library(verbose=True)
    build_probe(verbose=True)
