"""Host-side checks of bench.py's command line (no GPU): more than one GPU is refused with a message, and the
workloads it offers are the benchmark configurations."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
    assert not [l for l in r.stdout.splitlines() if l.startswith("{")]      # no result line


def test_workloads_offered_are_the_benchmark_configurations():
    sys.path.insert(0, ROOT)
    from paper_2602_12675_amd import workloads as W
    w = W.CONFIGS["wan1.3b-97-fp8"]
    assert (w.B, w.H, w.N, w.d, w.block_q, w.block_kv) == (1, 12, 32760, 128, 128, 64)
    assert abs(w.topk_frac - 0.03) < 1e-12 and w.quant == "fp8"
    w = W.CONFIGS["wan14b-97-fp8"]
    assert (w.B, w.H, w.N, w.d) == (1, 40, 75600, 128)
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "--workload" in r.stdout and "--steps" in r.stdout and "--warmup" in r.stdout
