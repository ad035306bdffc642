"""Compile the C oracle into oracle/libpalsgd_oracle.so with gcc.

The oracle is test infrastructure (see palsgd_oracle.c); building it is not
using it.  -O2, no hand vectorisation, OpenMP only for the static split of the
element loops.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "palsgd_oracle.c")
OUT = os.path.join(HERE, "libpalsgd_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= os.path.getmtime(SRC):
        return OUT
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-ffp-contract=off", "-o", OUT, SRC, "-lm"]
    subprocess.check_call(cmd)
    return OUT


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
