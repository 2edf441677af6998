"""The library driven from plain C (tests/c_abi_driver.c: HIP runtime + include/distattn.h, no Python in the path)."""
import os
import subprocess

import pytest

from paper_2401_02669_amd import build as hip_build

pytestmark = pytest.mark.gpu


def test_c_program_runs_the_path_and_matches_its_own_reference():
    exe = hip_build.C_DRIVER
    if not os.path.exists(exe):
        hip_build.build_c_driver()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "c abi driver: ok" in r.stdout
