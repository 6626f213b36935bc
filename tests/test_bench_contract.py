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


import json

import pytest


@pytest.mark.gpu
def test_result_line_carries_the_required_objects():
    """One short run on the benchmark workload: a single JSON line with the metric, the roofline of the
    attention kernel and the oracle's time on the host cores."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "4", "--warmup", "2", "--cpu-heads", "1",
                        "--no-backward"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 4 and d["warmup"] == 2 and d["vs_baseline"] is None
    assert d["config"]["workload"] == "wan1.3b-97-fp8" and d["data"] == "synthetic" and d["dtype"] == "fp8"
    assert abs(d["value"] - 4.0 * 32760 ** 2 * 128 * 12 / (d["ms_per_step"] * 1e-3) / 1e12) / d["value"] < 1e-3
    roof = d["roofline"]
    assert roof["bound"] in ("hbm", "mfma") and roof["unit"] in ("GB/s", "TFLOP/s")
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3 and 0 < roof["frac"] < 1
    assert roof["traffic"] is None or roof["traffic"] > 0
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
    # the same loop timed again at the end of the run is reported next to `value`, never as it
    settled = d["settled"]
    assert settled["steps"] == 4 and settled["ms_per_step"] > 0 and "order" in d and d["order"].startswith("W warm-up + K timed calls = value")
    assert roof["traffic_source"].startswith("profiles/")
    assert 0 < d["step_ms"]["min"] <= d["step_ms"]["median"] <= d["step_ms"]["max"]
    assert d["dense_bf16"]["ms"] > d["ms_per_step"] and abs(d["speedup_vs_dense_bf16"] - d["dense_bf16"]["ms"] / d["ms_per_step"]) < 0.02 * d["speedup_vs_dense_bf16"]
