"""Build the CPU oracle shared library (test infrastructure only).

Plain gcc, -O2, OpenMP; deliberately not tuned beyond that.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "gemm_oracle.c")
SOURCES = [SRC, os.path.join(HERE, "conv_oracle.c"), os.path.join(HERE, "level3_oracle.c")]
HEADERS = [os.path.join(HERE, "half_bits.h")]
LIB = os.path.join(HERE, "libgemm_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(f) for f in SOURCES + HEADERS):
        return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-o", LIB] + SOURCES + ["-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
