"""Compile the C oracle into oracle/liborc.so with gcc (test infrastructure)."""

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "tbs_oracle.c")
LIB = os.path.join(HERE, "liborc.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(
            os.path.getmtime(SRC), os.path.getmtime(os.path.join(HERE, "tbs_oracle.h"))):
        return LIB
    cmd = ["gcc", "-O3", "-std=c11", "-Wall", "-Wextra", "-fopenmp", "-shared", "-fPIC",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
    sys.exit(0)
