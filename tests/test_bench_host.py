"""Host-side behaviour of bench.py that needs no GPU: one GPU only, and argument checking."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_formula():
    # rows read x N x sizeof(w) + the inputs + fused bias + outputs (the per-unit figure the roofline uses)
    sys.path.insert(0, ROOT)
    import bench
    K, N = 14336, 4096
    assert bench.algorithmic_bytes(K, K, N, 1, 2) == K * N * 2 + K * 2 + N * 4 + N * 4
    assert bench.algorithmic_bytes(100, K, N, 16, 2) == 100 * N * 2 + 16 * K * 2 + N * 4 + 16 * N * 4
    assert bench.HBM_PEAK_GBS == 8000.0
