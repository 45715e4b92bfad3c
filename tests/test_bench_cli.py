"""Host-side checks of bench.py that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_measured_traffic_matches_the_committed_counter_summary():
    """The HBM bytes bench.py reports for the streaming kernel are the ones derived in profiles/."""
    sys.path.insert(0, ROOT)
    import bench
    text = open(os.path.join(ROOT, "profiles", "bench_resnet50_hbm_counters.md")).read()
    assert "HBM traffic per launch = %d bytes" % bench.MEASURED_TRAFFIC_BYTES in text
    assert bench.BYTES_PER_ENTRY == 12 and bench.HBM_PEAK_GBS == 8000.0
