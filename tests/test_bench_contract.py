"""bench.py's command-line contract that can be checked without a GPU."""

import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_of_the_headline_workload():
    sys.path.insert(0, ROOT)
    import bench
    # bf16 in + 4-bit codes + 16-bit metadata per block of 32: 2.5625 B per element
    assert bench.algorithmic_bytes(16384, 3072) == 128974848
    assert bench.algorithmic_bytes(16384, 3072, 16) == 16384 * 3072 * 2 + 16384 * 3072 // 2 + 16384 * 192 * 2
    assert bench.HBM_PEAK_GBS == 8000.0
