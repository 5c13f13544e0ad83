"""The device tables without a device.  The host parts of the library are built with g++ against a
synchronous stand-in for the HIP runtime, and kernel launches go to a CPU interpreter of the piece and hint
tables (tests/hostonly/cpu_kernels.cpp) that walks workgroups, wavefront tiles and lanes as the kernels do,
checks every address a kernel would touch against the buffers of the call, and moves the bytes (conversion
by the oracle).  tests/hostonly/table_cases.py then runs, in a child process on that build, random files,
ragged rows, rows shorter than a chunk, thousands of small tensors, every layout (resident, slot, packed,
sparse, compacted) and the stager, each against the oracle."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_23072_amd", "csrc")
HOSTONLY = os.path.join(ROOT, "tests", "hostonly")
HIP_INCLUDE = "/opt/rocm/include"


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir(HIP_INCLUDE), reason="g++ and the HIP headers needed")
def test_tables_on_the_cpu_interpreter(tmp_path):
    lib = str(tmp_path / "libfst_cpu.so")
    orc_o = str(tmp_path / "fst_oracle.o")
    subprocess.check_call(["gcc", "-O2", "-fPIC", "-c", os.path.join(ROOT, "oracle", "fst_oracle.c"), "-o", orc_o])
    subprocess.check_call(["g++", "-std=c++17", "-O2", "-g", "-fPIC", "-shared", "-pthread", "-w", "-D__HIP_PLATFORM_AMD__",
                           "-I", HIP_INCLUDE, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", os.path.join(ROOT, "oracle"),
                           os.path.join(CSRC, "header.cpp"), os.path.join(CSRC, "plan.cpp"),
                           "-x", "c++", os.path.join(CSRC, "stage.hip"), os.path.join(CSRC, "materialize.hip"), "-x", "none",
                           os.path.join(HOSTONLY, "fake_hip_sync.cpp"), os.path.join(HOSTONLY, "cpu_kernels.cpp"),
                           os.path.join(HOSTONLY, "static_stub.cpp"), orc_o, "-o", lib])
    env = dict(os.environ, FST_LIBRARY=lib)
    r = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
                        os.path.join(HOSTONLY, "table_cases.py")], cwd=ROOT, env=env, capture_output=True, text=True,
                       timeout=1500)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out[-6000:]
