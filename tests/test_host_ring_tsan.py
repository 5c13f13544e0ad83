"""The staging ring's host code under ThreadSanitizer, without a GPU: the sources of the ring, the
table builder, the parser and the planner are compiled with g++ -fsanitize=thread against a stand-in
for the HIP calls they make (streams = worker threads that run their queues in order; a kernel launch =
a queue entry that touches the launch's source and output buffers), and a driver stages a synthetic
file through tiny ring slots with several reader threads, resident and streamed.  A missing event wait
(a ring slot refilled before its copy ran, a device slot overwritten before its kernels ran) would show
as a data race."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_23072_amd", "csrc")
HOSTONLY = os.path.join(ROOT, "tests", "hostonly")
HIP_INCLUDE = "/opt/rocm/include"


def _has_tsan():
    p = subprocess.run(["gcc", "-print-file-name=libtsan.so"], capture_output=True, text=True).stdout.strip()
    return os.path.isabs(p) and os.path.exists(p)


@pytest.mark.skipif(shutil.which("g++") is None or not _has_tsan() or not os.path.isdir(HIP_INCLUDE),
                    reason="g++ with libtsan and the HIP headers needed")
def test_staging_ring_under_thread_sanitizer(tmp_path):
    exe = str(tmp_path / "ring_tsan")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=thread", "-fno-omit-frame-pointer", "-pthread",
                           "-w", "-D__HIP_PLATFORM_AMD__", "-I", HIP_INCLUDE, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                           os.path.join(CSRC, "header.cpp"), os.path.join(CSRC, "plan.cpp"),
                           "-x", "c++", os.path.join(CSRC, "stage.hip"), os.path.join(CSRC, "materialize.hip"), "-x", "none",
                           os.path.join(HOSTONLY, "fake_hip_streams.cpp"), os.path.join(HOSTONLY, "ring_main.cpp"), "-o", exe])
    for _ in range(3):          # thread interleavings differ from run to run
        r = subprocess.run([exe], capture_output=True, text=True, timeout=120,
                           env=dict(os.environ, TSAN_OPTIONS="halt_on_error=0 exitcode=66"))
        out = r.stdout + r.stderr
        assert "ThreadSanitizer" not in out, out[-6000:]
        assert r.returncode == 0 and out.strip().endswith("ok"), out[-2000:]
