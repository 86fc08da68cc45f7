"""Compile the CPU oracle (test infrastructure) into oracle/libminikv_ref.so with gcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(HERE, f) for f in ("minikv_ref.c", "minikv_pt_ref.c")]
HDRS = [os.path.join(HERE, f) for f in ("minikv_ref.h", "minikv_pt_ref.h")]
LIB = os.path.join(HERE, "libminikv_ref.so")

# -ffp-contract=off and no fast-math: the code decisions are individually rounded binary32 operations.
FLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC",
         "-Wall", "-Wextra"]


def build(force=False):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(f) for f in SRCS + HDRS):
        return LIB
    subprocess.check_call(["gcc", *FLAGS, *SRCS, "-o", LIB, "-lm"])
    return LIB


if __name__ == "__main__":
    print(build(force=True))
