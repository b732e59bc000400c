"""Compiles the CPU oracle (plain C, gcc) into oracle/libneuzip_oracle.so.

The oracle is test infrastructure: building it is not using it.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libneuzip_oracle.so")


def build(verbose: bool = False) -> str:
    src = os.path.join(HERE, "neuzip_oracle.c")
    cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-Wall", "-Wextra", "-pthread",
           "-o", LIB, src, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
