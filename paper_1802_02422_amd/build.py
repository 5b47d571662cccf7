"""Builds the HIP library in-tree with hipcc for gfx950."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "ivf_gp.hip")
LIB = os.path.join(HERE, "libivf_gp.so")

# packed fp32 VALU instructions are switched off for every HIP translation unit
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_library(verbose: bool = False) -> str:
    cmd = [os.environ.get("HIPCC", "hipcc"), *HIPCC_FLAGS, "-o", LIB, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd, stderr=None if verbose else subprocess.DEVNULL)
    return LIB


if __name__ == "__main__":
    build_library(verbose=True)
