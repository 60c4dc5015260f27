"""Builds libnoloco.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_2506_10911_amd.build

hipcc cross-compiles without a GPU. Flags that matter:
  -ffp-contract=off        every binary32 operation of the outer step rounds on its own
  -packed-fp32-ops off     no packed-fp32 instructions are generated (a device-code feature: it is
                           given only to the translation unit that holds device code)
"""
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OUT = os.path.join(PKG, "libnoloco.so")
OBJ = os.path.join(PKG, "_build")
HOST_SOURCES = ["api.cpp", "planner.cpp", "launch_plan.cpp", "latency_model.cpp"]   # no device code
DEVICE_SOURCES = ["kernels.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ROCM = os.path.dirname(os.path.dirname(os.path.realpath(HIPCC)))
COMMON = ["-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fno-fast-math", "-Wall",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC]
NO_PACKED_FP32 = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# hipcc compiles a .hip file twice, for the GPU and for the host; the host pass does not know the
# GPU feature above and says so once per file. That one line is dropped, everything else is shown.
HARMLESS = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"


def commands():
    cmds = []
    objs = []
    for src in HOST_SOURCES:
        obj = os.path.join(OBJ, src + ".o")
        objs.append(obj)
        # plain C++ that calls the HIP runtime API: compiled for the host only
        cmds.append([HIPCC, *COMMON, "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROCM, "include"), "-x", "c++", "-c", os.path.join(CSRC, src), "-o", obj])
    for src in DEVICE_SOURCES:
        obj = os.path.join(OBJ, src + ".o")
        objs.append(obj)
        cmds.append([HIPCC, "--offload-arch=gfx950", *COMMON, *NO_PACKED_FP32,
                     "-Wno-unused-command-line-argument", "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj])
    cmds.append([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", OUT])
    return cmds


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    for cmd in commands():
        if verbose:
            print(" ".join(cmd), flush=True)
        done = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
        noise = [l for l in done.stderr.splitlines() if l.strip() and HARMLESS not in l]
        if noise:
            print("\n".join(noise), file=sys.stderr, flush=True)
        if done.returncode != 0:
            raise subprocess.CalledProcessError(done.returncode, cmd)
    return OUT


if __name__ == "__main__":
    build()
    sys.exit(0)
