"""The host planner compiled with g++ -fsanitize=address,undefined and driven over many mask shapes
(no GPU: the device side is stubbed).  A memory error or undefined behaviour aborts the driver."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_planner_is_clean_under_address_and_ub_sanitizers(tmp_path):
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "planner_sanitizer_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-static-libasan", "-static-libubsan",  # (the runtimes are part of the executable: no load-order concerns)
           "-fno-omit-frame-pointer", "-pthread", "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(ROOT, "paper_2506_06095_amd", "csrc"),
           os.path.join(ROOT, "tests", "planner_sanitizer_driver.cpp"),
           os.path.join(ROOT, "paper_2506_06095_amd", "csrc", "plan.cpp"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "sanitize" in build.stderr and "cannot find" in build.stderr:
        pytest.skip("sanitizer runtime not installed")
    assert build.returncode == 0, build.stderr[-2000:]
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert run.returncode == 0, (run.stdout[-1000:], run.stderr[-3000:])
    assert "plans built and exported under the sanitizers" in run.stdout
