"""Compile the CPU oracle (test infrastructure) into oracle/libbagua_oracle.so with gcc.

No -march flags: the library built here is also run on the GPU machine's host CPU.
-ffp-contract=off and the absence of -ffast-math are part of the oracle's definition
(every written fp32 operation rounds once).
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "bagua_oracle.c")
LIB = os.path.join(HERE, "libbagua_oracle.so")

FLAGS = ["-std=c11", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
         "-fno-unsafe-math-optimizations", "-frounding-math", "-fsignaling-nans", "-Wall", "-Wextra"]


def build(force=True):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc"] + FLAGS + [SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
