"""Host-side checks of bench.py's command-line contract (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _load_bench():
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_model_flops_formula():
    import als_inputs as I
    b = _load_bench()
    w = I.workload("lm20m")
    L, d, S, V = w["L"], w["d"], w["S"], w["V"]
    # with attention width d and FFN width 4 d the general count is the textbook 24 d^2 one
    assert b.flops_per_token(w) == 3.0 * (L * (24.0 * d * d + 2.0 * S * d) + 2.0 * d * V)
    p = I.workload("paper150m_b128")
    a = p["h"] * p["dh"]
    per_layer = 2 * p["d"] * 3 * a + 2 * a * p["d"] + 2 * 2 * p["d"] * p["ff"] + 2 * p["S"] * a
    assert b.flops_per_token(p) == 3.0 * (p["L"] * per_layer + 2.0 * p["d"] * p["V"])


def test_peaks_are_the_published_ones():
    b = _load_bench()
    assert b.PEAK_BF16_TFLOPS == 2500.0 and b.PEAK_HBM_GBS == 8000.0
