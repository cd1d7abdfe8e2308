"""Host-side checks of bench.py's contract that need no GPU: more than one GPU is refused
with a message, and the committed counter summary carries the lines bench.py reads."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_summary_is_readable():
    sys.path.insert(0, ROOT)
    import bench
    per_launch = bench.read_traffic_note("C4a")
    per_step = bench.read_traffic_note("C4a", "traffic_bytes_per_step")
    algorithmic = 12.0 * 32 * 25_557_032
    assert algorithmic <= per_launch <= 1.1 * algorithmic
    assert per_launch <= per_step <= 1.2 * algorithmic
    assert bench.read_traffic_note("no-such-workload") is None
