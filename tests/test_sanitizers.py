"""AddressSanitizer + UndefinedBehaviorSanitizer over the CPU-side code: the oracle and the
library's host-only entry points, compiled with g++ into one small program and run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_oracle_and_host_code_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2504_12285_amd", "csrc"),
           os.path.join(ROOT, "tests", "sanitize_driver.cpp"),
           os.path.join(ROOT, "oracle", "bitlinear_oracle.cpp"),
           os.path.join(ROOT, "paper_2504_12285_amd", "csrc", "bl_api.cpp"), "-o", exe]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    assert run.returncode == 0 and "sanitizer run ok" in run.stdout, run.stdout
