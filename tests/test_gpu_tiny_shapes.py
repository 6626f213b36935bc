"""Shapes at and below one block: every kernel clamps its rows to the tokens that exist, the router ranks
one to three key blocks, and one of the two branches may be empty (one key block: it is either selected or
not).  Parity against the oracle in every precision mode."""
import numpy as np
import pytest

from helpers import check_mask, oracle_heads, rel_l2, rows_ok, run_forward
from paper_2602_12675_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = {"none": 2e-2, "fp8": 5e-2, "int8": 5e-2, "fp8v": 5e-2}


def tiny(N, dtype, quant, d, bq, topk):
    return W.TINY.replace(name="N%d-%s-%s-d%d-bq%d-k%g" % (N, dtype, quant, d, bq, topk), grid=(1, 1, N), H=2, d=d,
                          block_q=bq, dtype=dtype, quant=quant, topk_frac=topk, per_head_freq=True)


CASES = [tiny(N, dt, qm, d, bq, topk)
         for N in (1, 63, 65, 130)
         for (dt, qm, d, bq) in (("f32", "none", 64, 64), ("bf16", "none", 128, 128), ("bf16", "fp8", 128, 128),
                                 ("bf16", "int8", 64, 64), ("bf16", "fp8v", 128, 64))
         for topk in (0.5,)]
CASES += [tiny(65, "bf16", "fp8", 128, 128, 0.0), tiny(65, "bf16", "none", 128, 128, 1.0), tiny(1, "f32", "none", 64, 64, 0.0)]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_tiny_shapes_match_oracle(w):
    import torch
    from paper_2602_12675_amd import api
    inp = W.generate(w)
    r = run_forward(api, torch, inp)
    ref = oracle_heads(inp)
    for (b, h), o in ref.items():
        assert check_mask(r["idx"][b, h], o["R"], o["sel"]) == 0
        if w.dtype == "f32":
            np.testing.assert_allclose(r["out"][b, h], o["O"], rtol=0, atol=2e-3)
        else:
            assert rel_l2(r["out"][b, h], o["O"]) <= TOL[w.quant], (b, h)
            rows_ok(r["out"][b, h], o["O"], w.quant)
        fin = np.isfinite(o["L"])
        np.testing.assert_allclose(r["lse"][b, h][fin], o["L"][fin], rtol=0, atol=3e-2)
        assert np.all(np.isneginf(r["lse"][b, h][~fin]))
    assert np.isfinite(r["out"]).all()


@pytest.mark.parametrize("dtype,quant,d,bq", [("f32", "none", 64, 64), ("bf16", "none", 128, 128), ("bf16", "fp8", 128, 128),
                                              ("bf16", "none", 64, 64)])
@pytest.mark.parametrize("N", [961, 1983])
def test_all_but_one_block_selected(N, dtype, quant, d, bq):
    """k = T_n - 1 with a one-token (N = 961, T_n = 16) or 63-token (N = 1983, T_n = 31) last key block: the linear
    branch of a query block is what one key block leaves of the per-head totals.  The kernels form it by
    subtraction (totals minus the selected blocks), so this is where cancellation would show - for the
    query blocks whose left-out block is the one-token one, Z_i is one K^phi row against a total of 961."""
    import torch
    from paper_2602_12675_amd import api
    T_n = -(-N // 64)
    w = W.TINY.replace(name="k%d-of-%d-%s-%s" % (T_n - 1, T_n, dtype, quant), grid=(1, 1, N), H=3, d=d, block_q=bq,
                       dtype=dtype, quant=quant, topk_frac=(T_n - 1) / T_n, per_head_freq=True)
    assert w.k == T_n - 1
    inp = W.generate(w)
    r = run_forward(api, torch, inp)
    ref = oracle_heads(inp)
    left_out_last = 0
    for (b, h), o in ref.items():
        assert check_mask(r["idx"][b, h], o["R"], o["sel"]) == 0
        left_out_last += int(sum(T_n - 1 not in row for row in o["sel"].tolist()))
        if w.dtype == "f32":
            np.testing.assert_allclose(r["out"][b, h], o["O"], rtol=0, atol=2e-3)
        else:
            assert rel_l2(r["out"][b, h], o["O"]) <= TOL[w.quant], (b, h)
            rows_ok(r["out"][b, h], o["O"], w.quant)
    print("%s: query blocks whose linear branch is the short last block alone: %d" % (w.name, left_out_last))
    assert np.isfinite(r["out"]).all()
