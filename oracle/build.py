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
    # ORACLE_SANITIZE=undefined | address | address,undefined: a second library built with gcc's sanitizers (stops at
    # the first finding), which the wrapper then loads instead; the pins run against it in
    # tests/test_oracle_sanitized.py.  An address-sanitized library needs the sanitizer's runtime loaded first
    # (LD_PRELOAD of `gcc -print-file-name=libasan.so`); that test arranges it.
    san = os.environ.get("ORACLE_SANITIZE", "")
    lib, flags = LIB, FLAGS
    if san:
        lib = os.path.join(HERE, "liboracle_%s.so" % san.replace(",", "_"))
        flags = [f for f in FLAGS if f != "-O2"] + ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=" + san,
                                                     "-fno-sanitize-recover=all"]
    stale = (not os.path.exists(lib)) or os.path.getmtime(lib) < os.path.getmtime(SRC)
    if force or stale:
        tmp = lib + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *flags, SRC, "-o", tmp, "-lm"])
        os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    print(build(force=True))
