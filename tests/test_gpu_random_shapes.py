"""A seeded sample of the parameter space (token count, heads, batch, head dimension, block size, kept
fraction, precision mode, per-block alpha, smoothing on/off): GPU against the oracle.  The cases are fixed
by the seed; each is small enough for the oracle to finish in a fraction of a second."""
import numpy as np
import pytest

from helpers import check_mask, oracle_heads, rel_l2, rows_ok, run_forward
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
            rows_ok(r["out"][b, h], o["O"], w.quant)
        fin = np.isfinite(o["L"])
        np.testing.assert_allclose(r["lse"][b, h][fin], o["L"][fin], rtol=0, atol=3e-2)
    assert np.isfinite(r["out"]).all()


def draw_backward_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for c in range(n):
        dtype, quant = [("bf16", "none"), ("bf16", "fp8"), ("f32", "none"), ("bf16", "none")][c % 4]
        N = int(rng.integers(1, 2600))                       # up to 41 key blocks: more than one 32-column mask word
        topk = float(rng.choice([0.0, 1.0, rng.uniform(0.02, 0.5), rng.uniform(0.02, 0.5), rng.uniform(0.02, 0.5)]))
        w = W.TINY.replace(name="rndbwd%02d-N%d-%s-%s" % (c, N, dtype, quant), grid=(1, 1, N), B=int(rng.integers(1, 3)),
                           H=int(rng.integers(1, 4)), d=int(rng.choice([64, 128])), block_q=int(rng.choice([64, 128])),
                           dtype=dtype, quant=quant, topk_frac=topk, seed=int(rng.integers(0, 1 << 30)), per_head_freq=True)
        cases.append((w, bool(rng.integers(0, 2)), bool(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("w,per_block,smooth", draw_backward_cases(16, seed=2027),
                         ids=lambda x: x.name if hasattr(x, "name") else str(int(x)))
def test_random_configuration_backward_matches_oracle(w, per_block, smooth):
    import torch
    import sla2_oracle as O
    from paper_2602_12675_amd import api
    from test_gpu_backward import rel, run_fwd_bwd
    inp = W.generate(w)
    rng = np.random.default_rng(w.seed + 1)
    alpha = rng.uniform(0.05, 0.95, size=(w.H, w.T_m) if per_block else (w.H,)).astype(np.float32)
    dout = rng.normal(size=(w.B, w.H, w.N, w.d)).astype(np.float32)
    if w.dtype == "bf16":
        dout = W.f32_to_bf16_bits(dout)
    r = run_fwd_bwd(api, torch, inp, alpha, per_block, smooth, dout)
    assert all(np.isfinite(r[n]).all() for n in ("dq", "dk", "dv", "dalpha"))
    oq = {"none": O.QUANT_NONE, "fp8": O.QUANT_FP8}[w.quant]
    dal_ref = np.zeros(alpha.shape, dtype=np.float64)
    for b in range(w.B):
        for h in range(w.H):
            Q, K, V = (inp.values(n, b, h) for n in ("q", "k", "v"))
            g = O.backward_head(Q, K, V, r["idx"][b, h], alpha[h].astype(np.float64), r["go"][b, h].astype(np.float64),
                                w.block_q, w.block_kv, smooth=smooth, quant=oq)
            dal_ref[h] += g["dalpha"] if per_block else g["dalpha"].sum()
            for name in ("dq", "dk", "dv"):
                want = g["d" + name[1].upper()]
                if w.dtype == "f32":
                    np.testing.assert_allclose(r[name][b, h], want, rtol=0, atol=2e-4 * max(1.0, np.abs(want).max()),
                                               err_msg="%s b%d h%d" % (name, b, h))
                else:
                    scale = max(np.linalg.norm(want), 1e-3 * np.sqrt(want.size))   # all-zero gradients (k = T_n, alpha -> dV only)
                    assert np.linalg.norm(r[name][b, h] - want) <= 2e-2 * scale, (name, b, h, rel(r[name][b, h], want))
    if w.dtype == "f32":
        np.testing.assert_allclose(r["dalpha"], dal_ref, rtol=1e-4, atol=1e-3)
    else:
        np.testing.assert_allclose(r["dalpha"], dal_ref, rtol=3e-2, atol=3e-2 * max(np.abs(dal_ref).max(), 1e-3))
