"""Compile the C oracle into oracle/liboracle_cdsgd.so with gcc.

Test infrastructure: the flags keep IEEE fp32 semantics exactly as written in
the source (no fast-math, no contraction of multiply-add, no vectoriser tricks
that could reorder).
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "cdsgd_oracle.c")
LIB = os.path.join(HERE, "liboracle_cdsgd.so")

CFLAGS = ["-std=c11", "-O2", "-fno-fast-math", "-ffp-contract=off", "-fno-tree-vectorize",
          "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.run(["gcc", *CFLAGS, SRC, "-o", tmp, "-lm"], check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
