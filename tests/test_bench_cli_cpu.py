"""bench.py's command line without a GPU: more than one GPU is refused with a message, and the
roofline arithmetic (algorithmic bytes per launch) matches the per-token figures."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, cwd=ROOT)
    assert res.returncode != 0
    assert "one GPU" in (res.stdout + res.stderr)


def test_algorithmic_bytes():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    fwd, bwd = bench.algorithmic_bytes(75600, 5120, 2)
    assert fwd == 75600 * (4 * 5120 + 8) == 1548892800          # x in, y out, two float32 statistics
    assert bwd == 75600 * (6 * 5120 + 8) == 2323036800          # dy, x in, dx out, statistics in
    assert bench.PEAK_HBM_GBS == 8000.0
