"""Compile the CPU oracle (plain C) into oracle/libxq_oracle.so with gcc.

Test infrastructure: nothing in the product path builds or loads this.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "xq_oracle.c")
LIB = os.path.join(HERE, "libxq_oracle.so")

FLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
         "-fno-fast-math", "-ffp-contract=off", "-Wall", "-Wextra"]


def build(force=False):
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= os.path.getmtime(SRC)):
        return LIB
    cmd = ["gcc", *FLAGS, SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
