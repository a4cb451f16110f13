"""The transform schedule (csrc/wht_plan.h) checked on the host: csrc/plan_selftest.cpp is compiled
with g++ and verifies, for every configuration the library instantiates, that each butterfly stage
runs exactly once, that every layout is a bijection, that LDS addresses stay inside the token's
region, and -- by emulating the phases on the CPU -- that the schedule computes H_raw x."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2603_08343_amd", "csrc")


def test_schedule_selftest(tmp_path):
    exe = str(tmp_path / "plan_selftest")
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-o", exe,
                    os.path.join(CSRC, "plan_selftest.cpp")], check=True)
    out = subprocess.run([exe], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout
    lines = [l for l in out.stdout.splitlines() if " n=" in l]
    # butterfly schedule: float32 d = 2^5..2^13, bfloat16 d = 2^5..2^14; matrix-core: d = 2^10..2^14
    assert len(lines) == 9 + 10 + 5 and all(l.endswith(" ok") for l in lines), out.stdout
    assert sum(l.startswith("mfma") for l in lines) == 5
