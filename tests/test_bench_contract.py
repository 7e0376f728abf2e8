"""Host-side checks of bench.py's contract that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       cwd=ROOT, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_match_the_per_linear_table():
    # decode linear: codes C*N/2 + fp16 scale and 4-bit zero per (group, row) + X + Y
    # (+ 8 B per pair and 2 B per channel of transform parameters when fused)
    sys.path.insert(0, ROOT)
    import bench
    assert bench.algorithmic_bytes(4096, 6144, 1) == 13_234_176
    assert bench.algorithmic_bytes(4096, 4096, 1) == 8_871_936
    assert bench.algorithmic_bytes(4096, 28672, 1) == 61_218_816
    assert bench.algorithmic_bytes(14336, 4096, 1) == 31_031_296
    assert bench.algorithmic_bytes(4096, 28672, 1, rotated=False) < bench.algorithmic_bytes(4096, 28672, 1)
