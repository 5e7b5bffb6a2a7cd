"""The C oracle and the host build of the GPU lanes' construction code under AddressSanitizer and
UndefinedBehaviorSanitizer (host code only): both are compiled with -fsanitize=address,undefined into one small
driver (tests/sanitize_driver.cpp) that runs them over every p up to 160, a few larger p and single rows of the
largest p, and compares them with each other.  Any report ends the driver with a non-zero status."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
FLAGS = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


def test_oracle_and_lane_code_under_asan_and_ubsan(tmp_path):
    if shutil.which("gcc") is None or shutil.which("g++") is None:
        pytest.skip("no host compiler")
    obj = str(tmp_path / "oracle.o")
    exe = str(tmp_path / "driver")
    subprocess.run(["gcc", "-c"] + FLAGS + ["-o", obj, os.path.join(ROOT, "oracle", "bcs_oracle.c")], check=True)
    subprocess.run(["g++", "-std=c++17", "-Wno-unknown-pragmas"] + FLAGS +
                   ["-I", os.path.join(ROOT, "paper_2205_10072_amd", "csrc"), "-o", exe,
                    os.path.join(HERE, "bcs_hostcheck.cpp"), os.path.join(HERE, "sanitize_driver.cpp"), obj], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe, "160"], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert "sanitize_driver: ok" in run.stdout
