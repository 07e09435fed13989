"""Compile the C oracle into oracle/libsgemm_oracle.so with gcc.  Building the checker is not
using it: the product library neither links nor loads the result."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libsgemm_oracle.so")
SRC = [os.path.join(HERE, "sgemm_oracle.c")]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and all(
        os.path.getmtime(LIB) >= os.path.getmtime(s) for s in SRC
    ):
        return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-Wall", "-Wextra",
           "-o", LIB] + SRC
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
