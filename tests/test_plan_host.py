"""Host logic of the launch planning (csrc/plan.hpp has no HIP dependency): invariants over a sweep
of sizes -- every plan fits the workspace the ABI asks for, covers all rows, stays within LDS --
and the shapes chosen for the benchmark configurations.  Compiled with the host compiler."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_plan_invariants(tmp_path):
    cxx = shutil.which("g++") or shutil.which("c++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / "host_plan_check")
    src = os.path.join(ROOT, "tests", "host_plan_check.cpp")
    subprocess.run([cxx, "-std=c++17", "-O1", "-I", os.path.join(ROOT, "paper_2605_27390_amd", "csrc"), src, "-o", exe],
                   check=True)
    out = subprocess.run([exe], capture_output=True, text=True)
    assert out.returncode == 0 and out.stdout.strip() == "ok", out.stdout + out.stderr
