"""Compile the HIP library (csrc/wht_affine.hip) for gfx950 into libwht_affine.so, in-tree.

hipcc cross-compiles without a GPU.  Run as `python -m paper_2603_08343_amd.build`.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "wht_affine.hip")
LIB = os.path.join(HERE, "libwht_affine.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed float32 VALU forms are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # matrix-core results are consumed by vector ALU code: have them written to VGPRs directly
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = False, extra=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *extra, "-o", LIB, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def ensure_built(verbose: bool = False) -> str:
    """For harnesses (tests, smoke check, benchmark): compile only if nothing has been built yet.
    The binding itself never builds: a missing library is an error there."""
    if not os.path.exists(LIB):
        build(verbose=verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
