"""Builds tests/host_fuzz.cpp (the HIP-free host logic under a randomised driver) with
AddressSanitizer and UndefinedBehaviorSanitizer and runs it for several seeds.  CPU only."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_host_logic_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "host_fuzz")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-static-libasan", "-static-libubsan",
                    os.path.join(HERE, "host_fuzz.cpp"), "-o", exe], check=True)
    for seed in range(1, 9):
        res = subprocess.run([exe, str(seed), "250"], capture_output=True, text=True)
        assert res.returncode == 0, res.stdout + res.stderr
        assert "host fuzz ok" in res.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_background_planner_under_tsan(tmp_path):
    exe = str(tmp_path / "planner_thread_check")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=thread", "-static-libtsan", "-pthread",
                    os.path.join(HERE, "planner_thread_check.cpp"), "-o", exe], check=True)
    res = subprocess.run([exe], capture_output=True, text=True)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "planner threads ok" in res.stdout and "ThreadSanitizer" not in res.stderr
