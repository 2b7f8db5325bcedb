"""Compile oracle/atb_oracle.c into oracle/liboracle.so with gcc.

Deliberately plain flags: no fast-math, no FMA contraction, no -march=native
(the shared object is built on one machine and run on another).
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "atb_oracle.c")
OUT = os.path.join(HERE, "liboracle.so")


def build(verbose: bool = False) -> str:
    cmd = ["gcc", "-std=c99", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fno-fast-math", "-Wall", "-Wextra", "-o", OUT, SRC, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return OUT


def ensure_built() -> str:
    """Path of the shared object; builds it first if it is missing or older than its source."""
    if not os.path.exists(OUT) or os.path.getmtime(SRC) > os.path.getmtime(OUT) or \
            os.path.getmtime(os.path.abspath(__file__)) > os.path.getmtime(OUT):
        build()
    return OUT


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
