"""Host logic of the tuned kernels: the LDS address maps in thc_layout14.h are
bijections, writer and reader of every exchange agree on every coordinate's address,
and the access patterns are bank-conflict free under the documented bank model.
The check is a small C++ program (tests/layout_check.cpp) compiled with g++."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_lds_address_maps(tmp_path):
    exe = str(tmp_path / "layout_check")
    src = os.path.join(ROOT, "tests", "layout_check.cpp")
    inc = os.path.join(ROOT, "paper_2407_01378_amd", "csrc")
    subprocess.run(["g++", "-O1", "-std=c++17", f"-I{inc}", "-o", exe, src], check=True)
    res = subprocess.run([exe], stdout=subprocess.PIPE, text=True)
    assert res.returncode == 0, res.stdout
    assert "0 problems" in res.stdout
