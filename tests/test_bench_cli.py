"""bench.py is a one-GPU benchmark: asking for more GPUs must fail with a message, before any GPU work."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                          timeout=120)
    assert proc.returncode != 0
    assert "ONE GPU" in proc.stderr and proc.stdout.strip() == ""


def test_algorithmic_bytes_formula():
    """Per-rank algorithmic bytes: every activated slot's weights once + gathered x + act (write, then read) + y."""
    sys.path.insert(0, ROOT)
    import bench

    H, I, active, P = 7168, 2048, 35, 2101
    gu, dn = bench.algorithmic_bytes(active, P, H, I)
    assert gu == active * 2 * I * H * 2 + P * H * 2 + P * I * 2 + 4 * P
    assert dn == active * H * I * 2 + P * I * 2 + P * H * 2
    assert gu + dn == active * 3 * H * I * 2 + 2 * P * H * 2 + 2 * P * I * 2 + 4 * P
