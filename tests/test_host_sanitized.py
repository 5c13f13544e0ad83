"""The host parts of the library (header parser, load planner) rebuilt with g++ under AddressSanitizer
and UndefinedBehaviorSanitizer, and their tests run again on that build in a child process: hostile
headers and odd plans must not read out of bounds, overflow a signed integer or shift too far."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_23072_amd", "csrc")


def _runtime(name):
    p = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return p if os.path.isabs(p) and os.path.exists(p) else None


@pytest.mark.skipif(shutil.which("g++") is None or _runtime("libasan.so") is None, reason="g++ with libasan needed")
def test_parser_and_planner_under_asan_ubsan(tmp_path):
    lib = str(tmp_path / "libfst_hostonly.so")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-fno-omit-frame-pointer", "-fPIC", "-shared", "-pthread", "-I", os.path.join(ROOT, "include"),
                           "-I", CSRC, os.path.join(CSRC, "header.cpp"), os.path.join(CSRC, "plan.cpp"),
                           os.path.join(ROOT, "tests", "hostonly", "gpu_stubs.cpp"), "-o", lib])
    env = dict(os.environ, FST_LIBRARY=lib, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1",
               LD_PRELOAD=":".join(x for x in (_runtime("libasan.so"), _runtime("libubsan.so")) if x))
    # test_plan_errors also calls the launch half, which the stubs replace: left to the normal build
    r = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_host_parse.py"), os.path.join(ROOT, "tests", "test_host_plan.py"),
                        "--deselect", "tests/test_host_plan.py::test_plan_errors"],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    out = r.stdout + r.stderr
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
    assert r.returncode == 0, out[-4000:]
