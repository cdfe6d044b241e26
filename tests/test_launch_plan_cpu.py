"""Host logic of the launchers (shape tables, row plans, cost models) checked without a GPU: a small
C++ program includes csrc/lnmod_launch.hpp and walks every supported hidden size and 20 000 random
problems.  Needs only hipcc's host compiler."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_17923_amd", "csrc")


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if cand and os.path.exists(cand):
            return cand
    return None


def test_launch_plans_and_shape_tables(tmp_path):
    hipcc = _hipcc()
    if hipcc is None:
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "launch_plan_check")
    src = os.path.join(ROOT, "tests", "launch_plan_check.cpp")
    build = subprocess.run([hipcc, "-std=c++17", "-O1", "-I", CSRC, "-I", os.path.join(ROOT, "include"), src, "-o", exe],
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stdout + build.stderr
    run = subprocess.run([exe], capture_output=True, text=True)
    sys.stdout.write(run.stdout)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "0 failures" in run.stdout
