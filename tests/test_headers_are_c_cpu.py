"""The public headers are C: a C99 translation unit that includes all three compiles without
warnings, links against the built libraries and calls its host-side entry points (no GPU needed)."""
import os
import shutil
import subprocess

import pytest

from paper_2605_17923_amd import lnmod

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c_program_compiles_links_and_runs(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    if not os.path.exists(lnmod.LIBRARY):
        from paper_2605_17923_amd.build import build_library
        build_library()
    exe = str(tmp_path / "c_abi_check")
    libdir = os.path.dirname(lnmod.LIBRARY)
    build = subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                            os.path.join(ROOT, "tests", "c_abi_check.c"), "-o", exe, "-L", libdir, "-l:liblnmod.so", "-l:liblnmod_tools.so",
                            "-Wl,-rpath," + libdir], capture_output=True, text=True)
    assert build.returncode == 0, build.stdout + build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert run.returncode == 0, (run.returncode, run.stdout, run.stderr)
    assert "K=4 VPL=3 R=2 per_cu=1" in run.stdout
