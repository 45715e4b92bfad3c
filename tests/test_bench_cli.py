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


def test_traffic_is_read_from_the_committed_counter_summary():
    """The HBM bytes bench.py reports for the streaming kernel are parsed, at run time, from the
    counter summary under profiles/; the figure there follows from the table above it."""
    sys.path.insert(0, ROOT)
    import bench
    nbytes, kernel, source = bench.traffic_from_profile()
    text = open(os.path.join(ROOT, source)).read()
    assert kernel == "k_accumulate_filter" and source.startswith("profiles/")
    assert "HBM traffic per launch of %s = %d bytes" % (kernel, nbytes) in text
    # the derivation: (fetch KiB x fetch scale + write KiB x write scale) x 1024
    row = [c.strip() for c in next(l for l in text.splitlines() if l.startswith("| " + kernel)).split("|")]
    copy = [c.strip() for c in next(l for l in text.splitlines() if l.startswith("| k_copy_baseline")).split("|")]
    copy_kib = 25557032 * 4 / 1024.0
    fetch = float(row[3]) * copy_kib / float(copy[3])
    write = float(row[4]) * copy_kib / float(copy[4])
    assert abs((fetch + write) * 1024.0 - nbytes) <= 1e-3 * nbytes
    # at least the algorithmic bytes, and no wasted re-reads
    assert 12 * 25557032 <= nbytes <= 1.05 * 12 * 25557032
    assert bench.BYTES_PER_ENTRY == 12 and bench.HBM_PEAK_GBS == 8000.0


def test_cpu_baseline_legs_run_in_child_processes():
    """The oracle's two legs (one core, all usable cores) on a tiny model: same message bytes
    from both, core counts reported, children gone afterwards."""
    sys.path.insert(0, ROOT)
    import numpy as np
    import bench
    from paper_1805_08768_amd import synth
    sizes = [5000, 64, 20000, 300, 12000]
    host_sets = [synth.small_model_update(sizes, round_=r) for r in range(2)]
    pool = bench.CpuBaseline()
    try:
        out = pool.run(host_sets, sizes, 0.01, 1.0 / 32.0)
    finally:
        pool.close()
    one, every = out["legs"]
    assert one["cores"] == 1 and every["cores"] == min(len(sizes), len(os.sched_getaffinity(0)))
    assert out["cores"] == every["cores"] and out["usable_cores"] == len(os.sched_getaffinity(0))
    assert out["kind"] == "oracle" and out["unit"] == "elements/s" and out["value"] > 0
    # the per-tensor streams are independent of how the tensors are dealt out: the messages differ
    # only by the header and table entries of each share
    extra = (every["cores"] - 1) * 32 * 1.0
    assert abs(one["message_bytes_per_round"] + extra - every["message_bytes_per_round"]) < 1e-6
    assert all(not pr.is_alive() for pr, _ in pool.workers)
