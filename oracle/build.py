"""Compile the CPU oracle (plain C) into oracle/libsso.so.

Flags matter for bit-exactness: no FP contraction (so beta*m + (1-beta)*g is
two rounded products and one rounded sum, as the oracle's header states), no
fast-math.  OpenMP is only used by the multi-thread wrapper that the
benchmark's CPU baseline times.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "signsgd_oracle.c")
LIB = os.path.join(HERE, "libsso.so")

CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
          "-fno-fast-math", "-fopenmp", "-Wall", "-Wextra"]


def build(force=True):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, SRC])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
