"""The scorer's hand-counted waits (paper_2601_07891_amd/csrc/frag_schedule.h) against a model of
the in-order vector-memory queue: tests/host/frag_schedule_check.cpp, compiled here with g++
from the same header the kernel uses.  CPU only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "host", "frag_schedule_check.cpp")
INC = os.path.join(ROOT, "paper_2601_07891_amd", "csrc")


@pytest.fixture(scope="module")
def checker(tmp_path_factory):
    if shutil.which("g++") is None:
        pytest.skip("no host compiler")
    exe = str(tmp_path_factory.mktemp("frag") / "frag_schedule_check")
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-I", INC, SRC, "-o", exe], check=True)
    return exe


def test_no_operand_is_used_before_its_wait_has_covered_it(checker):
    r = subprocess.run([checker], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout
    # the counts are exact up to the load-to-LDS operations the hand-over leaves out
    assert "0 with an under-wait" in r.stdout


def test_a_count_one_too_large_is_caught(checker):
    # the planted mistake: every fragment wait allows one operation more
    r = subprocess.run([checker, "--plant"], capture_output=True, text=True)
    assert r.returncode == 1 and "used before it arrived" in r.stdout
