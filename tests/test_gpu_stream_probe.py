"""Runs the load-only streaming probe (tests/stream_probe.hip, built by tests/build_probe.py) and records what
HBM read rate the chip delivers for the attention kernel's address pattern and for its alternatives.  The
numbers go to a text file in the run's output folder; the assertions only say that the probe ran and that the ordering the
design relies on holds (heads of a block range on one XCD beat heads scattered over XCDs)."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_stream_probe_rates():
    exe = os.path.join(HERE, "stream_probe")
    if not os.path.exists(exe):
        import build_probe
        exe = build_probe.build(True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    rates = {}
    for line in res.stdout.strip().splitlines():
        name, us, gbs = line.split()
        rates[name] = (float(us), float(gbs))
    assert set(rates) == {"kernel-pattern", "heads-scattered", "plain-loads", "whole-blocks", "kernel-pattern-4096", "depth-3",
                          "head-pair", "head-quad", "head-quad-256", "head-quad-depth-3", "kv-adjacent"}
    for name, (us, gbs) in rates.items():
        assert 2000.0 < gbs < 8000.0, (name, gbs)              # plausible for 8 TB/s HBM3E, and below its peak
    assert rates["kernel-pattern"][1] > rates["heads-scattered"][1]
    os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
    with open(os.path.join(ROOT, "gpurun_out", "stream_probe.txt"), "w") as f:
        f.write(res.stdout)
