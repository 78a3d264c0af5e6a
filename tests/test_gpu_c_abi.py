"""The C ABI used from a plain C++ program (tests/c_abi/abi_smoke.cpp: hipMalloc'd buffers, no
Python, no torch in the process).  The build step compiles it against include/stream.h and the
shared library; this test runs it on the GPU (and builds it first if it is missing)."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_plain_cpp_caller(tmp_path):
    lib_dir = os.path.join(ROOT, "paper_2510_19875_amd")
    assert os.path.exists(os.path.join(lib_dir, "libstream_hip.so")), "build the library first"
    exe = os.path.join(ROOT, "tests", "c_abi", "abi_smoke")
    if not os.path.exists(exe):
        exe = str(tmp_path / "abi_smoke")
        hipcc = "/opt/rocm/bin/hipcc" if os.path.exists("/opt/rocm/bin/hipcc") else "hipcc"
        subprocess.check_call([hipcc, "-O1", "-std=c++17", "-I", os.path.join(ROOT, "include"),
                               os.path.join(ROOT, "tests", "c_abi", "abi_smoke.cpp"), "-o", exe,
                               "-L", lib_dir, "-lstream_hip", "-Wl,-rpath," + lib_dir])
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "c abi smoke ok" in r.stdout
