"""Builds the host-only sources with AddressSanitizer + UBSan (g++, no GPU code) and runs a seeded driver over the
work scheduler, the block pool and the placement scheduler."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2401_02669_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitizer_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-static-libasan", os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"),
           os.path.join(CSRC, "schedule.cpp"), os.path.join(CSRC, "block_pool.cpp"), os.path.join(CSRC, "placement.cpp"),
           "-o", exe]
    subprocess.check_call(cmd)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host sanitizer driver: ok" in r.stdout
