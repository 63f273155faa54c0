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


# XQ_ORACLE_SANITIZE=1 selects a second build of the same source with AddressSanitizer and
# UndefinedBehaviorSanitizer (any report aborts).  The CPU pins are run against it with the sanitizer
# runtime preloaded into the interpreter:
#   XQ_ORACLE_SANITIZE=1 ASAN_OPTIONS=detect_leaks=0 LD_PRELOAD="$LD_PRELOAD $(gcc -print-file-name=libasan.so)" \
#       python -m pytest tests -m "not gpu" -q
SAN_LIB = os.path.join(HERE, "libxq_oracle_san.so")
SAN_FLAGS = ["-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
             "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-Wall", "-Wextra"]


def sanitized():
    return os.environ.get("XQ_ORACLE_SANITIZE", "") == "1"


def build(force=False):
    lib, flags = (SAN_LIB, SAN_FLAGS) if sanitized() else (LIB, FLAGS)
    if (not force and os.path.exists(lib)
            and os.path.getmtime(lib) >= os.path.getmtime(SRC)):
        return lib
    cmd = ["gcc", *flags, SRC, "-o", lib, "-lm"]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
