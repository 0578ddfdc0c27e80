"""bench.py's command line, without a GPU: more than one GPU is refused with a message, and the
committed counter summaries carry the traffic figures that the JSON line reports."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_recorded_traffic_is_read_from_the_counter_summaries():
    sys.path.insert(0, ROOT)
    import bench
    for workload in ("citation", "social"):
        t = bench.recorded_traffic(workload)
        assert t is not None and 1e8 < t < 1e10
    assert bench.recorded_traffic("no such workload") is None
