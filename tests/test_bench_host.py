"""Host-side contract of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_of_the_headline_workload():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2510_20707_amd import synth
    wl = synth.WORKLOADS["c3"]
    # K and V once, the window queries, the kept rows read and written, the indices (bf16, D = 128, N = 8192, B = 64)
    per_unit = 2 * 8192 * 128 * 2 + 7 * 32 * 128 * 2 + 4 * 64 * 128 * 2 + 4 * 64
    assert bench.algorithmic_bytes(wl, 64, scores_out=False) == per_unit
    assert bench.algorithmic_bytes(wl, 64, scores_out=True) == per_unit + 4 * 8192
    assert bench.algorithmic_bytes(wl, 64, scores_out=False, reads_v=False) == per_unit - 8192 * 128 * 2
    assert per_unit * wl.n_units == 483553280
