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


@pytest.mark.skipif(not os.path.exists("/opt/rocm/bin/hipcc"), reason="hipcc not available")
def test_c_abi_host_side_under_asan_ubsan(tmp_path):
    """The whole library (host half instrumented, device half compiled as usual) driven through
    the C ABI in host-only mode by tests/api_fuzz.cpp; leak detection stays on."""
    exe = str(tmp_path / "api_fuzz")
    csrc = os.path.join(os.path.dirname(HERE), "paper_2601_10729_amd", "csrc")
    subprocess.run(["/opt/rocm/bin/hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-pthread",
                    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
                    "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                    "-Xarch_host", "-fno-sanitize-recover=all",
                    os.path.join(csrc, "orbit_kernels.hip"), os.path.join(csrc, "orbit_api.hip"),
                    os.path.join(HERE, "api_fuzz.cpp"), "-o", exe], check=True, capture_output=True)
    for seed in range(1, 9):
        res = subprocess.run([exe, str(seed), "400"], capture_output=True, text=True)
        assert res.returncode == 0, res.stdout[-1500:] + res.stderr[-3000:]
        assert "api fuzz ok" in res.stdout
