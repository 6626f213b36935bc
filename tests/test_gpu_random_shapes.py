"""A seeded sample of the parameter space (token count, heads, batch, head dimension, block size, kept
fraction, precision mode, per-block alpha, smoothing on/off): GPU against the oracle.  The cases are fixed
by the seed; each is small enough for the oracle to finish in a fraction of a second."""
import numpy as np
import pytest

from helpers import check_mask, oracle_heads, rel_l2, run_forward
from paper_2602_12675_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = {"none": 2e-2, "fp8": 5e-2, "int8": 5e-2, "fp8v": 5e-2}


def draw_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for c in range(n):
        dtype, quant = [("f32", "none"), ("bf16", "none"), ("bf16", "fp8"), ("bf16", "int8"), ("bf16", "fp8v")][c % 5]
        N = int(rng.integers(1, 1500))
        topk = float(rng.choice([0.0, 1.0, rng.uniform(0.02, 0.6), rng.uniform(0.02, 0.6), rng.uniform(0.02, 0.6)]))
        w = W.TINY.replace(name="rnd%02d-N%d-%s-%s" % (c, N, dtype, quant), grid=(1, 1, N), B=int(rng.integers(1, 3)),
                           H=int(rng.integers(1, 4)), d=int(rng.choice([64, 128])), block_q=int(rng.choice([64, 128])),
                           dtype=dtype, quant=quant, topk_frac=topk, seed=int(rng.integers(0, 1 << 30)), per_head_freq=True)
        cases.append((w, bool(rng.integers(0, 2)), bool(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("w,per_block,smooth", draw_cases(25, seed=2026), ids=lambda x: x.name if hasattr(x, "name") else str(int(x)))
def test_random_configuration_matches_oracle(w, per_block, smooth):
    import torch
    from paper_2602_12675_amd import api
    inp = W.generate(w)
    al = np.random.default_rng(w.seed).uniform(size=(w.H, w.T_m) if per_block else (w.H,)).astype(np.float32)
    r = run_forward(api, torch, inp, alpha=al, alpha_per_block=int(per_block), flags=0 if smooth else api.SLA2_FLAG_NO_SMOOTH_K)
    ref = oracle_heads(inp, alpha=al, smooth=smooth)
    for (b, h), o in ref.items():
        assert check_mask(r["idx"][b, h], o["R"], o["sel"]) == 0
        if w.dtype == "f32":
            np.testing.assert_allclose(r["out"][b, h], o["O"], rtol=0, atol=2e-3)
        else:
            assert rel_l2(r["out"][b, h], o["O"]) <= TOL[w.quant], (b, h)
        fin = np.isfinite(o["L"])
        np.testing.assert_allclose(r["lse"][b, h][fin], o["L"][fin], rtol=0, atol=3e-2)
    assert np.isfinite(r["out"]).all()
