"""Compile the C oracle into oracle/libsgemm_oracle.so with gcc.  Building the checker is not
using it: the product library neither links nor loads the result."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libsgemm_oracle.so")
SRC = [os.path.join(HERE, "sgemm_oracle.c")]
BASELINE_LIB = os.path.join(HERE, "libcpu_blocked_sgemm.so")
BASELINE_SRC = [os.path.join(HERE, "cpu_blocked_sgemm.c")]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and all(
        os.path.getmtime(LIB) >= os.path.getmtime(s) for s in SRC
    ):
        return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-Wall", "-Wextra",
           "-o", LIB] + SRC
    subprocess.run(cmd, check=True)
    return LIB


def build_baseline(force: bool = True) -> str:
    """The blocked fp32 CPU GEMM (a reported baseline, not the oracle): -O3, AVX2 + FMA."""
    if not force and os.path.exists(BASELINE_LIB) and all(
        os.path.getmtime(BASELINE_LIB) >= os.path.getmtime(s) for s in BASELINE_SRC
    ):
        return BASELINE_LIB
    cmd = ["gcc", "-O3", "-mavx2", "-mfma", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-Wall",
           "-Wextra", "-o", BASELINE_LIB] + BASELINE_SRC
    subprocess.run(cmd, check=True)
    return BASELINE_LIB


if __name__ == "__main__":
    print(build())
    print(build_baseline())
