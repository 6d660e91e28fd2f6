"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_byte_and_flop_formulas():
    """Algorithmic bytes and flops of one attention call as the measurement section defines them: K and V read
    once, Q read and O written once, parent read; 4*Hq*D flops per visible (query, key) pair."""
    sys.path.insert(0, ROOT)
    import bench
    L, N, Hq, Hkv, D = 8192, 64, 32, 8, 128
    assert bench.algorithmic_bytes(L, N, Hq, Hkv, D) == 4096 * (L + N) + 16384 * N + 4 * N
    assert bench.algorithmic_flops(L, N, Hq, D, depth_sum=100) == 4 * Hq * D * (N * L + 100)
    t, src = bench.measured_traffic(8192, 64)                    # the committed counter summary is found and parsed
    assert t is not None and t >= bench.algorithmic_bytes(L, N, Hq, Hkv, D)
    assert "profiles/" in src and "not measured by this run" in src
    assert bench.measured_traffic(1, 1) == (None, None)
