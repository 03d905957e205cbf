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


HEADER = os.path.join(ROOT, "include", "k2d.h")


LIB_TIMERS = os.path.join(HERE, "libk2d_timers.so")


def build(verbose=False, phase_timers=False):
    """Compiles the library; phase_timers=True builds the instrumented twin (libk2d_timers.so, compiled with
    -DK2D_PHASE_TIMERS: the step kernel records the clocks of its phases) that phase_timers.py uses."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + (["-DK2D_PHASE_TIMERS", "-o", LIB_TIMERS, SRC] if phase_timers else ["-o", LIB, SRC])
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed (exit %d):\n%s\n%s" % (r.returncode, r.stdout[-4000:], r.stderr[-8000:]))
    if verbose:
        print(r.stderr)
    return LIB_TIMERS if phase_timers else LIB


def stale():
    """True if the library is missing or older than its source or the header."""
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.exists(f) and os.path.getmtime(f) > t for f in (SRC, HEADER))


def ensure_built():
    """Path of the built library; rebuilds it when it is missing or older than k2d.hip / k2d.h (where no
    compiler is installed, a library that is there is used as it is)."""
    if stale():
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        if os.path.exists(LIB) and not os.path.exists(hipcc):
            return LIB
        build()
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
