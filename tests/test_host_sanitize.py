"""Host code of the library (planner, queries, policy, knobs) under
AddressSanitizer + UBSan: plan.cpp is plain C++ with no HIP dependency, so it is
built with g++ together with a small driver and run as a separate process."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_planner_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2311_04499_amd", "csrc"),
           os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"),
           os.path.join(ROOT, "paper_2311_04499_amd", "csrc", "plan.cpp"), "-o", exe]
    subprocess.check_call(cmd)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host sanitize driver: ok" in r.stdout
