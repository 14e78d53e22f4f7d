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


import json

import pytest


@pytest.mark.gpu
def test_bench_line_contract():
    """One short run of bench.py on the GPU: exactly one JSON line on stdout with the agreed fields."""
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--rank", "2", "--steps", "3", "--warmup", "1",
                           "--cpu-budget", "1", "--no-hip-graph"], capture_output=True, text=True, timeout=600)
    assert proc.returncode == 0, proc.stderr[-2000:]
    lines = [l for l in proc.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["unit"] == "GB/s" and d["value"] > 0
    assert d["config"]["workload"] == "deepseek_v3_decode" and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3 and 0 < r["frac"] < 1
    pc = d["per_config"]
    assert set(pc) == {"deepseek_v3_decode", "qwen3_235b_a22b_decode", "qwen3_30b_a3b_decode"}
    for cfg in pc.values():
        assert cfg["metro_vs_token_balanced"]["ffn_time_ratio"] > 0
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and c["unit"] == "GB/s" and c["sample"]
