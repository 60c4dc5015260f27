"""Builds libnoloco.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_2506_10911_amd.build

hipcc cross-compiles without a GPU. Flags that matter:
  -ffp-contract=off        every binary32 operation of the outer step rounds on its own
  -packed-fp32-ops off     no packed-fp32 instructions are generated
"""
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OUT = os.path.join(PKG, "libnoloco.so")
SOURCES = ["api.cpp", "planner.cpp", "launch_plan.cpp", "latency_model.cpp", "kernels.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def command():
    return [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
            "-ffp-contract=off", "-fno-fast-math",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wall", "-Wno-unused-command-line-argument",
            "-I", os.path.join(ROOT, "include"), "-I", CSRC,
            "-x", "hip", *[os.path.join(CSRC, s) for s in SOURCES],
            "-o", OUT]


def build(verbose: bool = True) -> str:
    cmd = command()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    build()
    sys.exit(0)
