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


def test_measured_traffic_record_is_read_from_the_profile_summary(tmp_path, monkeypatch):
    """The counter measurement is a number in a committed text summary, stamped with a hash of the kernel's sources:
    bench.py reports it only while those sources are what they were when it was taken."""
    sys.path.insert(0, ROOT)
    import bench
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    src = tmp_path / "paper_2503_00392_amd" / "csrc"
    src.mkdir(parents=True)
    for name in set(sum(bench.KERNEL_SOURCES.values(), [])):
        (src / name).write_text("// " + name)
    (tmp_path / "profiles").mkdir()
    stamp = bench.kernel_source_hash("select_kernel")
    (tmp_path / "profiles" / "hbm_traffic_w.md").write_text(
        "text\n`traffic_bytes_per_launch select_kernel = 411.5e6`\n`traffic_source_hash select_kernel = %s`\n" % stamp)
    v, st = bench.read_measured_traffic("w", "select_kernel")
    assert v == 411.5e6 and st["measured_at_source_hash"] == st["current_source_hash"] == stamp
    (src / "psa_select.hip").write_text("// changed")
    v, st = bench.read_measured_traffic("w", "select_kernel")
    assert v is None and st["measured_at_source_hash"] == stamp != st["current_source_hash"]
    assert bench.read_measured_traffic("w", "no_such_kernel")[0] is None
    assert bench.read_measured_traffic("no_such_workload", "select_kernel") == (None, None)


def test_the_committed_traffic_summary_parses():
    sys.path.insert(0, ROOT)
    import bench
    v, st = bench.read_measured_traffic("c3_128k_b4_l32", "select_kernel")
    assert st is not None and (v is None or 1.0e8 < v < 8.0e8)
