"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "ONE GPU" in p.stderr and p.stdout.strip() == ""


def test_measured_traffic_record_is_read_from_the_profile_summary():
    sys.path.insert(0, ROOT)
    import bench
    v = bench.read_measured_traffic("c3_128k_b4_l32", "select_kernel")
    assert v is not None and 3.0e8 < v < 6.0e8
    assert bench.read_measured_traffic("c3_128k_b4_l32", "no_such_kernel") is None
    assert bench.read_measured_traffic("no_such_workload", "select_kernel") is None
