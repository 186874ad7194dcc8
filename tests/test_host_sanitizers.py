"""The host half of the library under AddressSanitizer and UBSan (CPU only, g++).

Builds csrc/pool.cpp together with tests/host_fuzz.cpp into a sanitized executable and runs a
random workload over every host entry point.  Any sanitizer report or failed check fails the test.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_allocator_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "host_fuzz")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2503_18292_amd", "csrc"),
           os.path.join(ROOT, "paper_2503_18292_amd", "csrc", "pool.cpp"),
           os.path.join(ROOT, "tests", "host_fuzz.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", LD_PRELOAD="")
    for seed in (1, 2, 3):
        res = subprocess.run([exe, str(seed), "60000"], capture_output=True, text=True, env=env, timeout=300)
        assert res.returncode == 0, res.stdout + res.stderr
        assert "host_fuzz ok" in res.stdout
