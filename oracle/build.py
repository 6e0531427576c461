"""Compile the C oracle into a shared library next to its source.

Test infrastructure only: see the header of flex_oracle.c.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "flex_oracle.c")
LIB = os.path.join(HERE, "libflex_oracle.so")

# No fast-math, no contraction: every add is one IEEE binary32 operation.
CFLAGS = ["-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
          "-Wall", "-Wextra", "-shared", "-fPIC"]


def build(force: bool = False) -> str:
    stale = (not os.path.exists(LIB)
             or os.path.getmtime(LIB) < os.path.getmtime(SRC))
    if force or stale:
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, SRC, "-o", tmp])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
