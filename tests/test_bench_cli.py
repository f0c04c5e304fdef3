"""Host-side checks of bench.py's command line (no GPU)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "single-GPU" in r.stderr and r.stdout.strip() == ""


def test_model_flops_of_the_layer():
    """The flop count behind the reported TFLOP/s: the GPT-2-Medium-shaped layer at 50 % keep and dense (fwd+bwd, causal
    attention at half) - 335.0 and 670.0 GFLOP, twice the projection + FFN contractions plus the attention core."""
    sys.path.insert(0, ROOT)
    import bench
    T, L, d, h = 8192, 1024, 1024, 16
    sparse = bench.model_flops(T, L, d, h, 32, 32, 2048)
    dense = bench.model_flops(T, L, d, h, 64, 64, 4096)
    assert abs(sparse / 1e9 - 335.0) < 0.1 and abs(dense / 1e9 - 670.0) < 0.1 and abs(dense / sparse - 2.0) < 1e-12
    # shared key/value heads shrink only the K and V projections
    assert bench.model_flops(T, L, d, h, 64, 64, 4096, h_kv=4) < dense
