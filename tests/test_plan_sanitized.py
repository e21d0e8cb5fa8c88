"""The host-side launch planning (argument checks, key shares, row packing, workspace layout, the caps
that keep 32-bit offsets in range) compiled for the CPU alone under the address and undefined-behaviour
sanitizers and fuzzed over random and extreme shapes, strides and sizes (tests/plan_fuzz.cpp)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_planner_under_asan_and_ubsan(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no host C++ compiler")
    exe = tmp_path / "plan_fuzz"
    csrc = os.path.join(ROOT, "paper_2602_01053_amd", "csrc")
    build = subprocess.run(
        [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"), "-I", csrc,
         os.path.join(csrc, "lra_plan.cpp"), os.path.join(ROOT, "tests", "plan_fuzz.cpp"), "-o", str(exe)],
        capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([str(exe), "200000"], capture_output=True, text=True, timeout=300,
                         env=dict(os.environ, LD_PRELOAD="", ASAN_OPTIONS="detect_leaks=0"))
    assert run.returncode == 0, run.stdout + run.stderr
    assert "all plans consistent" in run.stdout
