"""The launch planner under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU: the planner is plain C++
(paper_2502_16982_amd/csrc/muon_plan.cpp, no HIP include), so it is built here with g++ alone together with a driver
that plans many shape lists, workspace budgets and arithmetics and walks every table the kernels would read."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_planner_is_clean_under_asan_and_ubsan(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("g++ not found")
    exe = str(tmp_path / "plan_sanitize")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-Wall", "-Wextra",
           os.path.join(ROOT, "paper_2502_16982_amd", "csrc", "muon_plan.cpp"),
           os.path.join(ROOT, "tests", "plan_sanitize_main.cpp"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stdout + build.stderr
    # verify_asan_link_order=0: the environment may preload libraries of its own ahead of the sanitizer runtime
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "planner ok" in run.stdout
