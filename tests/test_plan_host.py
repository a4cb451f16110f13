"""The transform schedule (csrc/wht_plan.h) checked on the host: csrc/plan_selftest.cpp is compiled
with g++ and verifies, for every configuration the library instantiates, that each butterfly stage
runs exactly once, that every layout is a bijection, that LDS addresses stay inside the token's
region, and -- by emulating the phases on the CPU -- that the schedule computes H_raw x; for rows
of 12 * 2^m elements, that the slot map is a bijection and that the padded schedule equals the
Kronecker definition."""
import os
import subprocess

import numpy as np

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2603_08343_amd", "csrc")


def test_schedule_selftest(tmp_path):
    exe = str(tmp_path / "plan_selftest")
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-o", exe,
                    os.path.join(CSRC, "plan_selftest.cpp")], check=True)
    out = subprocess.run([exe], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout
    lines = [l for l in out.stdout.splitlines() if " n=" in l]
    # butterfly schedule: float32 d = 2^5..2^13, bfloat16 d = 2^5..2^14; matrix-core: d = 2^10..2^14,
    # with separate forward and backward schedules at 2^14; rows of 12 * 2^m elements: d = 768..12288
    assert len(lines) == 9 + 10 + 6 + 5 and all(l.endswith(" ok") for l in lines), out.stdout
    assert sum(l.startswith("mfma") for l in lines) == 6
    assert sum(l.startswith("twelve") for l in lines) == 5
    # the order-12 factor the kernels carry (their own table) is the oracle's matrix
    out = subprocess.run([exe, "--p12"], capture_output=True, text=True, check=True)
    rows = out.stdout.split()
    table = np.array([[1 if c == "+" else -1 for c in row] for row in rows], dtype=np.int64)
    assert table.shape == (12, 12) and np.array_equal(table, oracle.h12())
