"""Compile the C oracle (test infrastructure) with gcc into oracle/libpccl_oracle.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "pccl_oracle.c")
LIB = os.path.join(HERE, "libpccl_oracle.so")

# No -ffast-math, no FMA contraction: every add must be one IEEE binary32 add.
CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
          "-fno-unsafe-math-optimizations", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    stale = (not os.path.exists(LIB)) or os.path.getmtime(LIB) < os.path.getmtime(SRC)
    if force or stale:
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, SRC, "-o", tmp])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
