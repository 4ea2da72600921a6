"""The parts of bench.py's contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


def test_bench_reads_the_committed_traffic_figures():
    sys.path.insert(0, ROOT)
    import bench
    import workloads
    for cfg in (4, 5):
        t, source = bench.measured_traffic(workloads.config(cfg).name)
        assert t is not None and t > 6.0e8, cfg          # HBM bytes per decode call from profiles/
        assert os.path.exists(os.path.join(ROOT, source))
    assert bench.measured_traffic("no_such_workload") == (None, None)
