"""Builds libtng.so for gfx950 with hipcc, in-tree (next to this file).

Flags that matter for reproducible codes: -ffp-contract=off keeps every fp32 operation of the
normalise / threshold / decode path a separately rounded IEEE operation (hipcc would otherwise
contract a*b+c into a fused multiply-add); no fast-math; correctly rounded division (the HIP
default); packed-fp32 instruction selection is switched off.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtng.so")
SOURCES = ["tng_api.hip", "tng_codec.hip", "tng_grad.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
]


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
