"""Compile the fp64 CPU oracle (plain C, OpenMP) into oracle/libdash_oracle.so.

Test infrastructure only: building the checker is not using it.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "dash_oracle.c")
LIB = os.path.join(HERE, "libdash_oracle.so")


def build_oracle(force: bool = True) -> str:
    """Compile dash_oracle.c with gcc. Baseline x86-64 code (no -march) so the
    library built in one container also runs on another machine."""
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
           SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build_oracle(force=True))
    sys.exit(0)
