"""The kernels' index arithmetic divides by multiplying with a reciprocal computed on the host (csrc/fast_div.h).
The helper is host-callable, so the host compiler builds a checker that compares it with the machine's division."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "..", "paper_2002_09539_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_reciprocal_division_matches_division(tmp_path):
    exe = str(tmp_path / "fast_div_check")
    subprocess.run(["g++", "-O1", "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + CSRC,
                    os.path.join(HERE, "host_fast_div_check.cpp"), "-o", exe], check=True)
    out = subprocess.run([exe], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout
    assert out.stdout.strip().endswith(" 0 mismatches")
