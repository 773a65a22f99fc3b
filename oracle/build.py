"""Compile the C oracle into oracle/liboracle.so with gcc.

Test infrastructure only (see dymoe_oracle.c).  Run as
``python -m oracle.build``; the Python wrapper also calls it when the
shared object is missing or older than its source.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "dymoe_oracle.c")
LIB = os.path.join(HERE, "liboracle.so")

# -ffp-contract=off: the quantizer is an exact sequence of binary32 operations.
FLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
         "-fPIC", "-shared"]


def build(force: bool = False) -> str:
    stale = (not os.path.exists(LIB)) or os.path.getmtime(LIB) < os.path.getmtime(SRC)
    if force or stale:
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *FLAGS, SRC, "-o", tmp, "-lm"])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
