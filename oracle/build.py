"""Compile the CPU oracle (plain C) into oracle/liboracle_gemm.so with gcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "oracle_gemm.c")
OUT = os.path.join(HERE, "liboracle_gemm.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= os.path.getmtime(SRC):
        return OUT
    # -O2 without -ffast-math: the summation order written in the source is kept.
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", OUT, SRC, "-lpthread", "-lm"]
    subprocess.check_call(cmd)
    return OUT


if __name__ == "__main__":
    print(build())
    sys.exit(0)
