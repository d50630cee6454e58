"""Builds the HIP library in-tree: ``python -m paper_2105_01827_amd.build``."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgala_hip.so")
SOURCES = ["gala_host.cpp", "gala_api.cpp", "gala_kernels.hip", "gala_perm2048.hip", "gala_conv_mfma.hip"]
HEADERS = ["gala_internal.h", "modarith.h", os.path.join("..", "..", "include", "gala.h")]
# packed-FP32 instructions are switched off for every device compile on the test machines
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread", "-Wno-unused-value", "-Wno-unused-command-line-argument",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(force=True, verbose=False):
    """Compile every source with hipcc for gfx950 into libgala_hip.so."""
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-o", LIB]
    for f in SOURCES:
        cmd += (["-x", "hip"] if f.endswith(".cpp") else []) + [os.path.join(CSRC, f)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build(force=True, verbose=True)
    print("built", LIB)
    sys.exit(0)
