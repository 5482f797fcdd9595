"""Builds libgns.so (HIP, gfx950 only) in-tree with hipcc."""
import glob
import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgns.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc_path():
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def build_library(verbose=False):
    """Compiles every csrc/*.hip into paper_2106_06150_amd/libgns.so.  Always recompiles."""
    sources = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    cmd = [hipcc_path()] + HIPCC_FLAGS + sources + ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
