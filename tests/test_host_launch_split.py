"""A launch class with more tiles than one dispatch can hold goes out as several dispatches, each told
the index of its first tile.  The cut and the workgroup -> tile permutation are plain host-compilable
functions of the library's internal header; a small g++ program checks that together they visit every
tile exactly once, for small limits exhaustively and for the real limit around its edges."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_23072_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ needed")
def test_launch_split_and_tile_permutation(tmp_path):
    exe = str(tmp_path / "split_main")
    subprocess.check_call(["g++", "-std=c++17", "-O2", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                           os.path.join(ROOT, "tests", "hostonly", "split_main.cpp"), "-o", exe])
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip() == "ok", r.stdout + r.stderr
