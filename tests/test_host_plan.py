"""The work split of the output projection is planned by one small function that the host (launch
sizes) and the kernels (with the row count they read on the device) both evaluate; the kernel that
merges the partials afterwards derives the number of partials from it again.  This test compiles
that function for the host and checks its properties; no GPU is involved."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_work_split_arithmetic_on_the_host(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "plan_check")
    cmd = [hipcc, "--cuda-host-only", "-std=c++17", "-O1", "-x", "hip",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2007_11794_amd", "csrc"),
           os.path.join(ROOT, "tests", "host", "plan_check.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip() == "ok", r.stdout[-2000:] + r.stderr[-2000:]
