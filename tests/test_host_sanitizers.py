"""The host-side code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU, no HIP): the
library's plan code (validation, sizes, tile tables of both chunk sizes and of plans with a bucket size
per layer), its bit-width assigners, and the CPU oracle are compiled with
`-fsanitize=address,undefined -fno-sanitize-recover=all` together with a small driver
(tests/host_sanitize/driver.cpp) that runs them on plans with every kind of layer and exactly sized
buffers, and the driver must exit cleanly."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2111_08617_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None or shutil.which("gcc") is None, reason="needs gcc and g++")
def test_plan_code_assigners_and_oracle_are_clean_under_asan_and_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    oracle_obj = str(tmp_path / "oracle.o")
    subprocess.run(["gcc", *san, "-std=c11", "-ffp-contract=off", "-c", os.path.join(ROOT, "oracle", "cgx_oracle.c"),
                    "-o", oracle_obj], check=True)
    exe = str(tmp_path / "driver")
    subprocess.run(["g++", *san, "-std=c++17", os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp"),
                    os.path.join(CSRC, "cgx_plan.cpp"), os.path.join(CSRC, "cgx_adaptive.cpp"), oracle_obj,
                    "-o", exe, "-lm"], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert "all checks passed" in run.stdout
