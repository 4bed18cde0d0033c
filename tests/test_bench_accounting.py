"""Host-side checks of bench.py: the byte accounting of the roofline line and the one-GPU rule (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench


def test_algorithmic_bytes_of_the_headline_shape():
    """d = d_v = 128, bf16, r = 0.75: keys read once 256 B, scores written once and read twice 12 B, a quarter of the
    indices 1 B, a quarter of the K and V rows read and written 2 x 0.25 x 512 = 256 B: 525 B per (head, token),
    4.95 GB for 36 x 8 x 32768 head-tokens."""
    ab = bench.algorithmic_bytes(128, 128, 2, 0.75)
    assert ab == {"scan": 256.0, "gather": 256.0, "total": 525.0}
    assert abs(ab["total"] * 36 * 8 * 32768 - 4.9545216e9) < 1.0


def test_algorithmic_bytes_of_other_shapes():
    assert bench.algorithmic_bytes(64, 64, 2, 0.5) == {"scan": 128.0, "gather": 256.0, "total": 398.0}
    ab = bench.algorithmic_bytes(128, 128, 2, 0.95)
    assert abs(ab["total"] - (256 + 12 + 0.2 + 51.2)) < 1e-9
    assert bench.algorithmic_bytes(128, 128, 1, 0.75)["scan"] == 128.0


def test_traffic_figure_is_read_from_the_committed_summary():
    t = bench.read_traffic("scan", "qwen4b_32k")
    assert t is not None and 2.4e9 < t < 3.0e9            # the keys once (2.416 GB) and a little more
    assert bench.read_traffic("scan", "no_such_workload") is None


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout == ""
