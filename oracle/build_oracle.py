"""Compile the plain-C oracles with gcc: oracle/tahq_oracle.c -> oracle/libtahq_oracle.so (the forward codec)
and oracle/naive_oracle.c -> oracle/libnaive_oracle.so (the backward fixed-point compressor).

Building the checker is not using it: the HIP library never links against it.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "tahq_oracle.c")
LIB = os.path.join(HERE, "libtahq_oracle.so")
NAIVE_SRC = os.path.join(HERE, "naive_oracle.c")
NAIVE_LIB = os.path.join(HERE, "libnaive_oracle.so")

# -ffp-contract=off: no a*b+c contraction; fmaf() is fused only where written.
CFLAGS = ["-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
          "-Wall", "-Wextra", "-Werror"]


def _compile(src, lib, force):
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(src):
        return lib
    subprocess.run(["gcc"] + CFLAGS + [src, "-o", lib, "-lm"], check=True)
    return lib


def build(force=True):
    _compile(NAIVE_SRC, NAIVE_LIB, force)
    return _compile(SRC, LIB, force)


if __name__ == "__main__":
    print(build())
    print(NAIVE_LIB)
