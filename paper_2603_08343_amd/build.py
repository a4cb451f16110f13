"""Compile the HIP library (csrc/wht_affine.hip) for gfx950 into libwht_affine.so, in-tree.

hipcc cross-compiles without a GPU.  Run as `python -m paper_2603_08343_amd.build`.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "wht_affine.hip")
LIB = os.path.join(HERE, "libwht_affine.so")
# bench-only object (a plain copy kernel): not part of the layer's ABI, never loaded by the binding
COPY_SRC = os.path.join(HERE, "csrc", "copy_bench.hip")
COPY_LIB = os.path.join(HERE, "libwht_copybench.so")
# debug build of the layer's library for one GPU test: after every LDS read the thread overwrites
# what it read with NaN, so that a read that comes before its data (a missing barrier or wait) shows
# up as NaN; carries the widths 512, 4096, 8192, 16384 and 6144 only
POISON_LIB = os.path.join(HERE, "libwht_affine_poison.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed float32 VALU forms are kept out of the generated code on the test machines.  The
    # feature belongs to the device target; the driver offers no way to pass a cc1 option to the
    # device pass alone, so the host pass sees it too and says it does not know it (filtered below).
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # matrix-core results are consumed by vector ALU code: have them written to VGPRs directly
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wall", "-Wno-unused-function",
]
SOURCES = [SRC] + [os.path.join(HERE, "csrc", f) for f in ("wht_device.h", "wht_plan.h")] + \
          [os.path.join(os.path.dirname(HERE), "include", "wht_affine.h")]


def build(verbose: bool = False, extra=()) -> str:
    _compile(COPY_SRC, COPY_LIB, verbose, extra)
    _compile(SRC, POISON_LIB, verbose, (*extra, "-DWHT_POISON_LDS"))
    return _compile(SRC, LIB, verbose, extra)


def _compile(src: str, lib: str, verbose: bool, extra=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *extra, "-o", lib, src]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    noise = "'-packed-fp32-ops' is not a recognized feature for this target"
    for line in proc.stderr.splitlines():
        if noise not in line:
            print(line, file=sys.stderr)
    if proc.returncode != 0:
        raise subprocess.CalledProcessError(proc.returncode, cmd)
    return lib


def ensure_built(verbose: bool = False) -> str:
    """For harnesses (tests, smoke check, benchmark): compile only if nothing has been built yet.
    The binding itself never builds: a missing library is an error there."""
    if not os.path.exists(LIB) or not os.path.exists(COPY_LIB) or not os.path.exists(POISON_LIB):
        build(verbose=verbose)
    elif any(os.path.getmtime(f) > min(os.path.getmtime(LIB), os.path.getmtime(POISON_LIB))
             for f in SOURCES if os.path.exists(f)):
        # a stale binary would be validated and recorded under the new sources' name
        raise RuntimeError(f"{LIB} is older than its sources: run `python -m paper_2603_08343_amd.build`")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
