"""Compile oracle/tahq_oracle.c into oracle/libtahq_oracle.so with gcc.

Building the checker is not using it: the HIP library never links against it.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "tahq_oracle.c")
LIB = os.path.join(HERE, "libtahq_oracle.so")

# -ffp-contract=off: no a*b+c contraction; fmaf() is fused only where written.
CFLAGS = ["-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
          "-Wall", "-Wextra", "-Werror"]


def build(force=True):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc"] + CFLAGS + [SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
