"""Compile the CPU oracle (plain C, gcc) into oracle/libjvoracle.so.

Test infrastructure: the product library never links or loads this.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "jvoracle.c")
OUT = os.path.join(HERE, "libjvoracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= os.path.getmtime(SRC):
        return OUT
    # -O3 for the timed baseline; the instruction set is pinned to the x86-64-v3 level (AVX2, FMA)
    # rather than to the build machine's own, because the library is built on one machine and
    # timed on another.
    cmd = ["gcc", "-std=c11", "-O3", "-march=x86-64-v3", "-fopenmp", "-shared", "-fPIC", "-Wall",
           "-Wextra", SRC, "-o", OUT, "-lm"]
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
