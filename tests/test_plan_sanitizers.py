"""The plan builder (host C++) under AddressSanitizer and UndefinedBehaviorSanitizer.

plan.cpp holds no GPU code, so it is compiled here with g++ together with a small driver
(tests/plan_sanitize.cpp) that builds fragments, descriptors and tiles for valid and invalid
shapes.  Any out-of-bounds access, signed overflow or leak aborts the driver."""

import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_plan_builder_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "plan_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan",  # no dependence on the order of preloaded libraries
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2507_19017_amd", "csrc"),
           os.path.join(ROOT, "paper_2507_19017_amd", "csrc", "plan.cpp"), os.path.join(ROOT, "tests", "plan_sanitize.cpp"),
           "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.strip().endswith("ok")
