"""The host planner under the host compiler's address and undefined-behaviour sanitizers.

The planner is plain C++ (no HIP runtime), so it is built here with g++ together with a small driver
(tests/planner_sanitizer_driver.cpp) that feeds it seeded random batches, valid and invalid, with
every tuning value, and checks each accepted plan's tables for bounds and exact coverage.  Any
out-of-bounds access, overflow or other undefined behaviour inside the planner aborts the driver.
"""
from __future__ import annotations

import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_planner_is_clean_under_address_and_ub_sanitizers(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / "planner_sanitized")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", os.path.join(HERE, "planner_sanitizer_driver.cpp"),
           os.path.join(ROOT, "paper_2410_18038_amd", "csrc", "pod_planner.cpp"), "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and ("cannot find -lasan" in built.stderr or "cannot find -lubsan" in built.stderr):
        pytest.skip("sanitizer runtimes are not installed")
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1")
    run = subprocess.run([exe, "600"], capture_output=True, text=True, env=env, timeout=300)
    if run.returncode != 0 and "ASan runtime does not come first" in run.stderr:
        pytest.skip("another preloaded library keeps the sanitizer runtime from starting")
    assert run.returncode == 0, run.stdout + run.stderr
    assert "plans checked" in run.stdout
    n_ok = int(run.stdout.split("sanitizers:")[1].split()[0])
    assert n_ok >= 400
