"""Compile the CPU oracle (oracle/wht_oracle.c) into oracle/libwht_oracle.so with gcc.

Test infrastructure only: nothing in the product path imports this.
Run as `python -m oracle.build`, or call `build()`.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "wht_oracle.c")
LIB = os.path.join(HERE, "libwht_oracle.so")


def build(verbose: bool = False) -> str:
    # plain -O2, no -ffast-math: IEEE double semantics are part of what the oracle is
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def ensure_built() -> str:
    if not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        build()
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
