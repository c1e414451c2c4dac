"""Host-side logic of the library that has no GPU in it, compiled and run on the CPU."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_scalar_division_constants_are_exact():
    """The kernels divide wave-uniform numbers by launch constants with one multiply-high and a shift
    (FastDiv); the constants the host prepares must give the exact quotient for every n < 2^31."""
    tmp = tempfile.mkdtemp(prefix="qnn_host_")
    try:
        exe = os.path.join(tmp, "fast_div")
        subprocess.run([HIPCC, "-O2", "-std=c++17", "-x", "hip", "--cuda-host-only",
                        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2106_09886_amd", "csrc"),
                        os.path.join(ROOT, "tests", "host_fast_div.cpp"), "-o", exe], check=True,
                       stdout=subprocess.PIPE, stderr=subprocess.PIPE)
        r = subprocess.run([exe], stdout=subprocess.PIPE, text=True)
        assert r.returncode == 0, r.stdout
        assert "bad 0" in r.stdout
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
