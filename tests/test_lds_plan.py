"""The streaming attention kernel reads its K / V^T fragments from LDS with hand-counted waits (csrc/lds_plan.h).
A host program replays the plan against an in-order queue: every wait must guarantee its fragment, be no stricter
than needed and fit the hardware counter, and no fragment register may be overwritten before its last use."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")
def test_lds_plan_replay(tmp_path):
    exe = tmp_path / "check_lds_plan"
    subprocess.run(["g++", "-std=c++17", "-O1", "-o", str(exe), os.path.join(HERE, "check_lds_plan.cpp")], check=True)
    run = subprocess.run([str(exe)], capture_output=True, text=True)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "lds plan ok" in run.stdout
