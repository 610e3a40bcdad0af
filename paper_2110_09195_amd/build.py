"""Build the HIP library for gfx950 with hipcc (cross-compiles without a GPU).

    python -m paper_2110_09195_amd.build [extra hipcc flags]

The shared objects are written next to this file (libsnn_hip.so, the product, and libsnn_peaks.so,
the measured-peak probes that bench.py runs) so that they travel with the source tree; nothing is installed.  Object files go to a temporary directory.
"""
import concurrent.futures
import os
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsnn_hip.so")
# the measured-peak probes of include/snn_peaks.h: a library of their own, loaded by bench.py only
PEAKS_LIB = os.path.join(HERE, "libsnn_peaks.so")
PEAKS_SOURCES = ["peaks.hip"]
SOURCES = ["snn_api.hip", "pack.hip", "project.hip", "bnn_conv.hip", "subbit_conv.hip", "subbit_f32.hip",
           "subbit_mfma.hip", "subbit_stack.hip", "train_ops.hip", "dense_fp4.hip"]

# Packed-fp32 VALU forms are switched off for all device code of this library.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]
# extra flags for tuning builds, e.g. SNN_BUILD_FLAGS="-DSNN_MF_TRACE"
FLAGS += os.environ.get("SNN_BUILD_FLAGS", "").split()


def build(verbose=False, extra=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory(prefix="snn_build_") as tmp:
        def compile_one(src):
            obj = os.path.join(tmp, src + ".o")
            cmd = [hipcc] + FLAGS + list(extra) + ["-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj

        with concurrent.futures.ThreadPoolExecutor(max_workers=8) as pool:
            objs = list(pool.map(compile_one, SOURCES + PEAKS_SOURCES))
        for lib, part in ((LIB, objs[:len(SOURCES)]), (PEAKS_LIB, objs[len(SOURCES):])):
            cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc"] + part + ["-o", lib]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
    print("built", LIB)
