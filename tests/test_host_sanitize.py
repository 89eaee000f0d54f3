"""The host-side bucket plan and ready tracker, compiled for the CPU with the
address and undefined-behaviour sanitizers and driven by a seeded random walk
(out-of-range and repeated ready marks included)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_plan_and_tracker_under_sanitizers(tmp_path):
    csrc = os.path.join(ROOT, "paper_2006_15704_amd", "csrc")
    exe = str(tmp_path / "plan_fuzz")
    build = subprocess.run(
        ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-I", csrc, "-o", exe, os.path.join(ROOT, "tests", "host_sanitize", "plan_fuzz.cpp"),
         os.path.join(csrc, "bucket_plan.cpp")],
        stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert run.returncode == 0 and run.stdout.strip().endswith("ok"), run.stdout
