"""The streaming attention kernel synchronises by hand: LDS fragment reads with counted waits, and a ring of K/V
stages filled by direct-to-LDS loads with counted waits and one barrier per two kblocks (csrc/lds_plan.h, which the
kernel compiles in).  Two host programs replay those plans:
  check_lds_plan.cpp   in-order LDS queue: every wait guarantees its fragment, is no stricter than needed, fits the
                       hardware counter; no fragment register is overwritten before its last use;
  check_ring_plan.cpp  waves under random interleavings, loads landing at random times: no read ever meets a stage
                       fragment that has not landed or may already be overwritten.
The ring checker is also run on copies of the plan with one constant changed, where it must report a violation."""
import os
import re
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
PLAN = os.path.join(HERE, "..", "paper_2509_22622_amd", "csrc", "lds_plan.h")

pytestmark = pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")


def _build_and_run(tmp_path, source, name):
    exe = tmp_path / name
    subprocess.run(["g++", "-std=c++17", "-O1", "-o", str(exe), str(source)], check=True)
    return subprocess.run([str(exe)], capture_output=True, text=True)


def test_lds_plan_replay(tmp_path):
    run = _build_and_run(tmp_path, os.path.join(HERE, "check_lds_plan.cpp"), "check_lds_plan")
    assert run.returncode == 0, run.stdout + run.stderr
    assert "lds plan ok" in run.stdout


def test_ring_plan_simulation(tmp_path):
    run = _build_and_run(tmp_path, os.path.join(HERE, "check_ring_plan.cpp"), "check_ring_plan")
    assert run.returncode == 0, run.stdout + run.stderr
    assert "ring plan ok" in run.stdout


@pytest.mark.parametrize("old, new", [
    ("AHEAD = 6", "AHEAD = 7"),                                   # a stage rewritten before its last read
    ("return step & 1;", "return (step & 3) == 3;"),              # barriers too far apart for 8 stages
    ("LANDED = 4", "LANDED = 3"),                                 # a pair of steps reads a kblock still in flight
    ("STAGES = 8", "STAGES = 4"),                                 # ring shorter than the loads run ahead
])
def test_ring_simulation_catches_a_wrong_plan(tmp_path, old, new):
    text = open(PLAN).read()
    assert old in text
    (tmp_path / "paper_2509_22622_amd" / "csrc").mkdir(parents=True)
    (tmp_path / "tests").mkdir()
    (tmp_path / "paper_2509_22622_amd" / "csrc" / "lds_plan.h").write_text(text.replace(old, new))
    shutil.copy(os.path.join(HERE, "check_ring_plan.cpp"), tmp_path / "tests" / "check_ring_plan.cpp")
    run = _build_and_run(tmp_path, tmp_path / "tests" / "check_ring_plan.cpp", "check_wrong")
    assert run.returncode == 1 and re.search(r"reads kblock \d+", run.stdout), run.stdout + run.stderr


def test_fp8_lds_plan_replay(tmp_path):
    """The 8-bit kernel's fragment reads (two slots ahead, four rotating buffers, one wait count for every slot)."""
    run = _build_and_run(tmp_path, os.path.join(HERE, "check_fp8_lds_plan.cpp"), "check_fp8_lds_plan")
    assert run.returncode == 0, run.stdout + run.stderr
    assert "fp8 lds plan ok" in run.stdout


@pytest.mark.parametrize("old, new, message", [
    ("return (AHEAD_SLOTS - 1) * READS_PER_FRAGMENT; }", "return (AHEAD_SLOTS - 1) * READS_PER_FRAGMENT + 1; }", "too weak"),
    ("static constexpr int AHEAD_SLOTS = 2;", "static constexpr int AHEAD_SLOTS = 3;", "rewritten"),
    ("static constexpr int buffer(int slot) { return slot % BUFFERS; }",
     "static constexpr int buffer(int slot) { return (slot + 1) % BUFFERS; }", None),
])
def test_fp8_plan_check_catches_a_wrong_plan(tmp_path, old, new, message):
    text = open(PLAN).read()
    assert old in text
    (tmp_path / "paper_2509_22622_amd" / "csrc").mkdir(parents=True)
    (tmp_path / "tests").mkdir()
    (tmp_path / "paper_2509_22622_amd" / "csrc" / "lds_plan.h").write_text(text.replace(old, new))
    shutil.copy(os.path.join(HERE, "check_fp8_lds_plan.cpp"), tmp_path / "tests" / "check_fp8_lds_plan.cpp")
    run = _build_and_run(tmp_path, tmp_path / "tests" / "check_fp8_lds_plan.cpp", "check_wrong")
    if message is None:                       # a consistent renaming of the buffers is still a correct plan
        assert run.returncode == 0, run.stdout + run.stderr
    else:
        assert run.returncode == 1 and message in run.stdout, run.stdout + run.stderr
