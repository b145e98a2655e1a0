"""Compile the CPU oracle (plain C, OpenMP) into oracle/libhalo_ref.so.

Test infrastructure: building the checker is not using it.  Run as
`python oracle/build.py` or through `__graft_entry__.build()`.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "halo_ref.c")
OUT = os.path.join(HERE, "libhalo_ref.so")


def build(verbose: bool = False) -> str:
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-shared", "-fPIC", "-Wall", "-Wextra", "-o", OUT, SRC, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return OUT


def ensure_built() -> str:
    if (not os.path.exists(OUT)) or os.path.getmtime(OUT) < os.path.getmtime(SRC):
        build()
    return OUT


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
