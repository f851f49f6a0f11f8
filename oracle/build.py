"""Compile the CPU oracle (plain C, gcc) into oracle/libmsd_oracle.so.

The oracle is test infrastructure: nothing in the product library links against it.
-ffp-contract=off keeps gcc from fusing a*b+c on its own, so the only fused operation
is the explicit fmaf() of the residual step.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "msd_oracle.c")
OUT = os.path.join(HERE, "libmsd_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= os.path.getmtime(SRC):
        return OUT
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra", "-shared", "-fPIC", SRC, "-o", OUT, "-lm"]
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
