"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only; the GPU code has no
sanitizer run): the CPU oracle (driven on exact-size heap buffers by oracle_sanitize_driver.c), the
schedule self-test that emulates every transform schedule, and the C ABI's argument validation."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2603_08343_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="4")
ENV.pop("LD_PRELOAD", None)          # the sanitizer runtime must come first in the link order


def _run(exe):
    out = subprocess.run([exe], capture_output=True, text=True, env=ENV)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "runtime error" not in out.stderr and "AddressSanitizer" not in out.stderr, out.stderr
    return out.stdout


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.run(["gcc", "-std=c11", "-fopenmp", "-Wall", "-Wextra", *SAN, "-o", exe,
                    os.path.join(ROOT, "tests", "oracle_sanitize_driver.c"),
                    os.path.join(ROOT, "oracle", "wht_oracle.c"), "-lm"], check=True)
    assert "oracle_sanitize_driver: ok" in _run(exe)


def test_schedule_selftest_under_sanitizers(tmp_path):
    exe = str(tmp_path / "plan_san")
    subprocess.run(["g++", "-std=c++17", "-Wall", *SAN, "-o", exe, os.path.join(CSRC, "plan_selftest.cpp")], check=True)
    out = _run(exe)
    lines = [l for l in out.splitlines() if " n=" in l]
    assert lines and all(l.endswith(" ok") for l in lines), out


def test_argument_validation_under_sanitizers(tmp_path):
    exe = str(tmp_path / "validate_san")
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", *SAN, "-o", exe,
                    os.path.join(CSRC, "validate_selftest.cpp")], check=True)
    assert "validate_selftest: ok" in _run(exe)
