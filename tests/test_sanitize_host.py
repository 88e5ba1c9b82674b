"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only): the dynamic-buffer
manager and candidate formation (csrc/arc.cpp), the launch planning (csrc/plan.hpp, the same sweep as
test_plan_host.py) and the CPU oracle (oracle/evospec_oracle.c), each driven by a small program that
replays seeded inputs through the C entry points.  Any finding aborts the program."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_27390_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
# (another preloaded library may come before the ASan runtime in the list: that order is not checked)
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
           UBSAN_OPTIONS="print_stacktrace=1")


def build_and_run(tmp_path, compiler, flags, sources, name):
    cc = shutil.which(compiler)
    if cc is None:
        pytest.skip(f"no {compiler}")
    exe = str(tmp_path / name)
    res = subprocess.run([cc, *flags, *SAN, *sources, "-o", exe], capture_output=True, text=True)
    if res.returncode != 0 and "sanitize" in res.stderr and "cannot find" in res.stderr:
        pytest.skip("the sanitizer runtimes are not installed")
    assert res.returncode == 0, res.stderr
    out = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=600)
    assert out.returncode == 0 and out.stdout.strip().endswith("ok"), out.stdout[-2000:] + out.stderr[-4000:]


def test_buffer_manager_and_candidates_under_sanitizers(tmp_path):
    build_and_run(tmp_path, "g++", ["-std=c++17", "-Wall", "-I", os.path.join(ROOT, "include")],
                  [os.path.join(CSRC, "arc.cpp"), os.path.join(ROOT, "tests", "host_sanitize_arc.cpp")], "san_arc")


def test_launch_planning_under_sanitizers(tmp_path):
    build_and_run(tmp_path, "g++", ["-std=c++17", "-I", CSRC], [os.path.join(ROOT, "tests", "host_plan_check.cpp")], "san_plan")


def test_oracle_under_sanitizers(tmp_path):
    build_and_run(tmp_path, "gcc", ["-std=c11", "-Wall", "-fopenmp"],
                  [os.path.join(ROOT, "oracle", "evospec_oracle.c"), os.path.join(ROOT, "tests", "host_sanitize_oracle.c"), "-lm"],
                  "san_oracle")
