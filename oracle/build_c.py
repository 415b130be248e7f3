"""Compile the oracle's plain-C CSR baseline (gcc, OpenMP) into oracle/libcsr_ref.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libcsr_ref.so")


def build(verbose: bool = False) -> str:
    cmd = ["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-std=c11",
           os.path.join(HERE, "csr_spmm_ref.c"), "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
