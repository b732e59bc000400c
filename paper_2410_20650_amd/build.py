"""Builds libneuzip.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
# NEUZIP_LIBRARY points the binding at another build of the library (tuning runs); build() always writes the in-tree one
LIB = os.environ.get("NEUZIP_LIBRARY") or os.path.join(HERE, "libneuzip.so")
BUILT_LIB = os.path.join(HERE, "libneuzip.so")
SOURCES = [os.path.join(HERE, "csrc", "neuzip.hip")]
HEADERS = [os.path.join(ROOT, "include", "neuzip.h")] + [
    os.path.join(HERE, "csrc", name)
    for name in ("neuzip_format.h", "neuzip_compress_kernels.h", "neuzip_decode_kernels.h",
                 "neuzip_linear_kernels.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Wall", "-Wno-unused-result",
    # packed fp32 instructions stay off for every HIP translation unit of this project
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def is_stale() -> bool:
    if not os.path.exists(BUILT_LIB):
        return True
    built = os.path.getmtime(BUILT_LIB)
    return any(os.path.getmtime(p) > built for p in SOURCES + HEADERS)


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), *SOURCES, "-o", BUILT_LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return BUILT_LIB


if __name__ == "__main__":
    build(verbose=True)
