"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/bapipe_oracle.c is
compiled with gcc -fsanitize=address,undefined together with a small C driver
(tests/oracle_sanitize_main.c) that calls every function on exactly-sized heap tensors; any
out-of-bounds access, signed overflow or misaligned access aborts the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-Wall", "-Wextra", "-o", exe,
           os.path.join(ROOT, "tests", "oracle_sanitize_main.c"), os.path.join(ROOT, "oracle", "bapipe_oracle.c"), "-lm"]
    subprocess.check_call(cmd)
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.returncode, r.stdout[-2000:], r.stderr[-4000:])
    assert "oracle sanitizer run clean" in r.stdout
