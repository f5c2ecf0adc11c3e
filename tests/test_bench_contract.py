"""Host-side checks of the benchmark's command line contract (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_algorithmic_bytes_of_the_headline_workload():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2310_02065_amd import inputs
    R, K, C, V, M, _ = inputs.CONFIGS["gpt3"]
    G = K // M
    # values 4 B per (row, group), metadata 4 bits, column-loc 8 B per (block row, group), B and C once
    assert bench.algorithmic_bytes(R, K, C, V, M) == 4 * R * G + R * G // 2 + 8 * (R // V) * G + 2 * K * C + 2 * R * C
    assert abs(bench.algorithmic_bytes(R, K, C, V, M) - 337.8e6) < 0.1e6
