"""The host-prepared division the MFMA kernel's index arithmetic uses (csrc/fastdiv.h), checked on the CPU:
the header is plain C++, so the same code the kernels compile is compiled here with g++."""
import os
import shutil
import subprocess

import pytest

from paper_2505_14687_amd.build import CSRC

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_fastdiv_equals_division(tmp_path):
    exe = tmp_path / "fastdiv_check"
    subprocess.run(["g++", "-O2", "-std=c++17", "-I", CSRC, os.path.join(HERE, "fastdiv_check.cpp"), "-o", str(exe)],
                   check=True)
    res = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.strip().endswith(" 0 bad"), res.stdout
