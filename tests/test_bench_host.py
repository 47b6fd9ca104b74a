"""Host-side checks of bench.py that need no GPU: the one-GPU contract of its command line, the
algorithmic byte count behind the roofline figure, and the key of the stored HBM traffic record."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
import synth  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "one GPU" in p.stderr and p.stdout.strip() == ""


def test_algorithmic_bytes_count_one_read_and_one_write_per_counted_row():
    w = synth.WORKLOADS["1p5b"]
    row = w.V * 2
    assert w.elem_bytes == 2 and w.T == 32768 and w.V == 151936
    # every row counted: read once + written once; no row counted: zero-filled once; side arrays 30 B per token
    assert bench.algorithmic_bytes(w, w.T) == 2 * row * w.T + 30 * w.T
    assert bench.algorithmic_bytes(w, 0) == row * w.T + 30 * w.T
    assert bench.algorithmic_bytes(w, 23550) == row * (2 * 23550 + (w.T - 23550)) + 30 * w.T == 17114446336


def test_traffic_record_is_keyed_by_the_kernel_sources():
    t = bench.measured_traffic("1p5b", "ragged")
    assert t is None or 0.99 < t / bench.algorithmic_bytes(synth.WORKLOADS["1p5b"], 23550) < 1.05
    assert bench.measured_traffic("no such workload", "ragged") is None
