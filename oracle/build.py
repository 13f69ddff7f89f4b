"""Compile the C oracle into ``oracle/libmmse_oracle.so`` (test infrastructure)."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "mmse_oracle.c")
OUT = os.path.join(_HERE, "libmmse_oracle.so")

# -ffp-contract=off: every fused multiply-add in the source is an explicit fmaf();
# nothing else may be fused.  -mfma/-msse4.1 only make fmaf()/rintf() inline.
CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-mfma", "-msse4.1", "-fopenmp",
          "-shared", "-fPIC", "-Wall", "-Wextra"]


def build(verbose: bool = False, src: str = SRC, out: str = OUT) -> str:
    cmd = ["gcc", *CFLAGS, src, "-o", out, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
