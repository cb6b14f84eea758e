"""Host logic behind the kernels: the LDS geometry that stage 1 bakes into the
candidate entries (which aligned place of which shifted row copy an entry
reads), its inverse, and the work classes.  The check itself is a small host
program, tests/host/geometry_check.cpp, which states every property from the
layout's definition; it is compiled for the host only and runs without a GPU."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_lds_geometry_and_work_classes(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = tmp_path / "geometry_check"
    build = subprocess.run(
        [hipcc, "-x", "hip", "--cuda-host-only", "-O1",
         "-I", os.path.join(ROOT, "include"),
         "-I", os.path.join(ROOT, "paper_2407_14843_amd", "csrc"),
         os.path.join(ROOT, "tests", "host", "geometry_check.cpp"), "-o", str(exe)],
        capture_output=True, text=True, timeout=300)
    assert build.returncode == 0, build.stderr[-2000:]
    run = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stdout[-2000:]
    assert "geometry ok" in run.stdout
