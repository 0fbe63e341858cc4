"""Compiles the C oracle (plain C, OpenMP over rows) into liboracle.so with gcc.

Run on the CPU, before anything touches a GPU: `python -m oracle.build`.  The digest of ppv_oracle.c is stamped
into the library, so that `oracle` can refuse a library that was built from another source."""
from __future__ import annotations

import hashlib
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ppv_oracle.c")
LIB = os.path.join(HERE, "liboracle.so")


def build_oracle(verbose: bool = True) -> str:
    with open(SRC, "rb") as f:
        digest = hashlib.sha256(f.read()).hexdigest()
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", f'-DORACLE_SOURCE_DIGEST="{digest}"', "-o", LIB,
           SRC, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build_oracle()
    sys.exit(0)
