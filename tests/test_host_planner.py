"""Builds the planner (host-only C++) with g++ under the address and undefined-behaviour
sanitizers and runs the coverage / bounds checker of tests/host_plan_check.cpp."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_planner_tiles_cover_and_stay_in_bounds(tmp_path):
    exe = str(tmp_path / "host_plan_check")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_1905_13727_amd", "csrc"),
           os.path.join(ROOT, "tests", "host_plan_check.cpp"),
           os.path.join(ROOT, "paper_1905_13727_amd", "csrc", "psgd_plan.cpp"), "-o", exe]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0 and "OK" in res.stdout, res.stdout
