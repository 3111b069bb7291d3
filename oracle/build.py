"""Compile the CPU oracle (test infrastructure) into oracle/liboracle.so.

The oracle is plain C built with gcc; `-ffp-contract=off` keeps the compiler
from fusing or reassociating anything the source does not spell out (the
distance recipes call fma() explicitly), `-mfma` only makes that fma() a
hardware instruction.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "knn_oracle.c")
LIB = os.path.join(HERE, "liboracle.so")


def build(force: bool = False) -> str:
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= os.path.getmtime(SRC)):
        return LIB
    cmd = ["gcc", "-std=gnu11", "-O2", "-mfma", "-fopenmp", "-ffp-contract=off",
           "-fPIC", "-shared", "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
