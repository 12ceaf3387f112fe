"""Build libmaxscore.so for gfx950 with hipcc (cross-compiles without a GPU)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmaxscore.so")
SOURCES = ["api.cpp", "solver.hip", "softtopk.hip", "dispatch.hip", "movement.hip", "iter.hip", "training.hip", "operators.hip", "alg1.hip", "sinkhorn.hip", "gemm.hip"]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-x", "hip",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", LIB] + os.environ.get("MAXSCORE_CXXFLAGS", "").split() + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
