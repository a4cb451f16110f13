"""The bfloat16 kernels exist in two schedules for d >= 1024: the matrix-core one (default, covered
by test_gpu_parity.py) and the all-butterfly one, selected per process by WHT_AFFINE_SCHEDULE.
This runs the parity check of the non-default schedule in a child process."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def test_butterfly_schedule_bf16_large_d():
    env = dict(os.environ, WHT_AFFINE_SCHEDULE="butterfly")
    print("[parity] butterfly schedule, bf16, d = 1024..16384 (child process)", flush=True)
    out = subprocess.run([sys.executable, os.path.join(HERE, "schedule_check.py")], env=env,
                         capture_output=True, text=True, timeout=280)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-2000:]
    assert "[schedule_check] ok" in out.stdout
