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


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    return bench


def test_traffic_comes_from_the_tracked_table_and_only_for_the_launch_it_was_measured_on(tmp_path, monkeypatch):
    from paper_2605_17923_amd import lnmod_tools
    bench = _bench()
    fwd = lnmod_tools.lnmod_describe_launch(False, None, 1, 75600, False, 5120, 0, 0)
    bwd = lnmod_tools.lnmod_describe_launch(True, None, 1, 75600, False, 5120, 0, 0)
    # the committed table describes today's launches of the headline workload
    f, b = bench.measured_traffic("forward", fwd), bench.measured_traffic("backward", bwd)
    fwd_alg, bwd_alg = bench.algorithmic_bytes(75600, 5120, 2)
    assert f is not None and fwd_alg <= f <= 1.01 * fwd_alg
    assert b is not None and bwd_alg <= b <= 1.03 * bwd_alg
    # another launch (other grid, other kernel instantiation) or another entry: no figure rather than a stale one
    assert bench.measured_traffic("forward", fwd.replace("grid=256", "grid=512")) is None
    assert bench.measured_traffic("forward", bwd) is None and bench.measured_traffic("backward", fwd) is None
    other = lnmod_tools.lnmod_describe_launch(False, (4, 3, 1, 2), 1, 75600, False, 5120, 0, 0)
    assert bench.measured_traffic("forward", other) is None
    table = tmp_path / "t.txt"
    table.write_text("# comment\nforward | some launch | 123 | abc | x.md\nbroken line\n")
    monkeypatch.setattr(bench, "TRAFFIC_TABLE", str(table))
    assert bench.measured_traffic("forward", "some launch") == 123
    assert bench.measured_traffic("forward", fwd) is None
    monkeypatch.setattr(bench, "TRAFFIC_TABLE", str(tmp_path / "missing.txt"))
    assert bench.measured_traffic("forward", "some launch") is None
