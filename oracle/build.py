"""Compile the C oracle into oracle/liboracle_sparse_attn.so (gcc, OpenMP, no fast-math).

Plain x86-64 code generation on purpose: the library is built in one container and
loaded on another machine, so no -march=native.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "sparse_attn_oracle.c")
LIB = os.path.join(HERE, "liboracle_sparse_attn.so")


def build(verbose: bool = False) -> str:
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
