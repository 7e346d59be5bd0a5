"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only).

tests/oracle_sanitizer_main.c walks Gen, Eval, the all-inputs sweep, the ReLU round and the window
unrolling over small ragged cases with every buffer allocated at its exact size; this test builds
it together with oracle/fss_oracle.c under the sanitizers and runs it as a child process.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not present")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-Wall", "-Wextra", "-fopenmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           os.path.join(ROOT, "tests", "oracle_sanitizer_main.c"), os.path.join(ROOT, "oracle", "fss_oracle.c"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "asan" in build.stderr.lower():
        pytest.skip("this gcc cannot link the sanitizer runtimes: " + build.stderr.strip().splitlines()[-1])
    assert build.returncode == 0, build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "oracle sanitizer walk: ok" in run.stdout
