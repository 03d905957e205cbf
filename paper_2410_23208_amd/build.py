"""Builds libk2d.so (the C-ABI library of include/k2d.h) for gfx950 with hipcc, in-tree."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "k2d.hip")
LIB = os.path.join(HERE, "libk2d.so")

# -ffp-contract=off: a*b+c is rounded twice, like a plain evaluation of the paper's formulas.
# -packed-fp32-ops is switched off on purpose (scalar fp32 VALU code only).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fPIC", "-shared", "-I" + os.path.join(ROOT, "include")]


def build(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-o", LIB, SRC]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL if not verbose else None,
                   stderr=subprocess.DEVNULL if not verbose else None)
    return LIB


def ensure_built():
    """Path of the built library; builds it only if it is missing."""
    if not os.path.exists(LIB):
        build()
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
