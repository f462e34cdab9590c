"""bench.py contract checks that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_table_names_every_workload():
    sys.path.insert(0, ROOT)
    import bench
    assert set(bench.TRAFFIC_BYTES) == {"c1", "c2", "c3", "c4", "c5", "g1", "g2", "m1", "m2", "m3", "a1", "a2", "l1"}
    assert bench.PEAK_BF16_TFLOPS == 2516.6 and bench.PEAK_HBM_GBS == 8000.0
