"""Compile the CPU oracle (test infrastructure) into oracle/libtao_oracle.so with gcc.

Flags matter: -frounding-math and -ffp-contract=off keep every operation a
separately rounded IEEE operation under the directed rounding mode the oracle
sets; no fast-math, no SIMD intrinsics.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "tao_oracle.c")
LIB = os.path.join(HERE, "libtao_oracle.so")

FLAGS = ["-O2", "-std=c11", "-frounding-math", "-ffp-contract=off", "-fno-fast-math",
         "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force=True):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc"] + FLAGS + [SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
