"""Build the HIP library for gfx950 with hipcc (cross-compiles without a GPU).

    python -m paper_2110_09195_amd.build

The shared object is written next to this file (libsnn_hip.so) so that it travels with the
source tree; nothing is installed.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsnn_hip.so")
SOURCES = ["snn_api.hip", "pack.hip", "project.hip", "bnn_conv.hip", "subbit_conv.hip", "subbit_f32.hip", "subbit_mfma.hip"]

# Packed-fp32 VALU forms are switched off for all device code of this library.
FAST = ["-DSNN_FAST_BUILD"] if os.environ.get("SNN_FAST_BUILD") else []
if os.environ.get("SNN_TUNE_BUILD"):
    FAST = ["-DSNN_FAST_BUILD"] + os.environ["SNN_TUNE_BUILD"].split()
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(verbose=False, extra=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + FAST + list(extra) + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
    print("built", LIB)
