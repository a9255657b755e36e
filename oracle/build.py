"""Compile the fp64 CPU oracle (test infrastructure) into oracle/libpbkv_oracle.so.

Plain gcc, -O2, no fast-math and no -march=native: the summation order stays
the one written in the source and the library runs on any x86-64 host.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "pbkv_oracle.c")
LIB = os.path.join(HERE, "libpbkv_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
           SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
