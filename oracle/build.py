"""Compiles the oracle (plain C++, host only) into oracle/_noloco_oracle.so.

Test infrastructure: nothing in the product path runs this file or loads its output.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "noloco_oracle.cpp")
OUT = os.path.join(HERE, "_noloco_oracle.so")

# -ffp-contract=off: the binary32 instantiation must round after every operation.
CMD = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math",
       "-shared", "-fPIC", "-o", OUT, SRC]


def build(verbose: bool = False) -> str:
    if verbose:
        print(" ".join(CMD), flush=True)
    subprocess.run(CMD, check=True)
    return OUT


def ensure_built() -> str:
    """Builds only when the library is absent or older than its source."""
    if not os.path.exists(OUT) or os.path.getmtime(OUT) < os.path.getmtime(SRC):
        build()
    return OUT


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
