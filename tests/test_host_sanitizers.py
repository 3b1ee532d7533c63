"""The host plan generator under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2007_12216_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_plan_generator_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "plan_sanitizer_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan",   # runtimes linked in: no dependence on the order of preloaded libraries
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(ROOT, "tests", "host", "plan_sanitizer_driver.cpp"), os.path.join(CSRC, "plan_math.cpp"), "-o", exe]
    build = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1"
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "bad=0" in run.stdout
