"""The host planner under AddressSanitizer + UndefinedBehaviorSanitizer: plan.cpp is pure host
C++, so it is built here with g++ and a small driver (tests/native/) and run over 3200 random
plans in every mode.  No GPU, no HIP."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_planner_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "plan_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan",   # runtime inside the executable: no library-order requirement
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2510_08874_amd", "csrc"),
           os.path.join(ROOT, "paper_2510_08874_amd", "csrc", "plan.cpp"),
           os.path.join(ROOT, "tests", "native", "plan_sanitize_driver.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert run.stdout.startswith("ok plans=3200")
