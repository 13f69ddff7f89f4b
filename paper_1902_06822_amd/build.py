"""Compile the HIP library for gfx950 into ``paper_1902_06822_amd/libmmse_hip.so``.

hipcc cross-compiles without a GPU.  Flags that matter for the result:
  -ffp-contract=off   every fused multiply-add in the kernels is written explicitly
  -fhip-fp32-correctly-rounded-divide-sqrt   IEEE fp32 division for the grid and 1/alpha
  -packed-fp32-ops disabled   no packed fp32 instructions are generated
"""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
SRC = [os.path.join(_HERE, "csrc", "mmse_kernels.hip")]
OUT = os.path.join(_HERE, "libmmse_hip.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17",
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-shared", "-fPIC", "-I" + os.path.join(ROOT, "include"),
]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *SRC, "-o", OUT]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
