"""GPU parity of the SoftTop-k router (Sec. 6) against the oracle's bisection, through the C ABI.
Both sides solve the same monotone equation in fp64 until the bracket stops shrinking; the masks
are float32 on the GPU side, so agreement is required to 1e-6 absolute and the row sums to k
within the float32 rounding of T_n entries."""
import numpy as np
import pytest

import sla2_oracle as O
from paper_2602_12675_amd import workloads as W

pytestmark = pytest.mark.gpu

CASES = [
    (W.TINY, 0.1),
    (W.TINY.replace(name="tiny-ragged", grid=(3, 11, 31)), 0.1),                                   # N = 1023
    (W.TINY.replace(name="bf16-d128", grid=(5, 16, 33), d=128, block_q=128, dtype="bf16", H=3,
                    topk_frac=0.1, per_head_freq=True), 0.1),                                       # N = 2640
    (W.TINY.replace(name="bf16-d64-wide", grid=(9, 30, 52), d=64, dtype="bf16", H=1, topk_frac=0.05), 0.02),  # T_n = 220
    (W.TINY.replace(name="bf16-d128-1200-blocks", grid=(24, 50, 64), d=128, block_q=128, dtype="bf16", H=1,
                    topk_frac=0.15, extra_tokens=3), 0.1),                                          # T_n = 1201
]


def run_soft(api, torch, inp, tau, topk_frac=None):
    w = inp.workload
    dt = api.SLA2_BF16 if w.dtype == "bf16" else api.SLA2_F32
    p = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac if topk_frac is None else topk_frac,
                        dtype=dt)
    q, k = api.to_device(inp.q, dt), api.to_device(inp.k, dt)
    rw = torch.from_numpy(inp.router_w).cuda()
    ws = api.alloc_workspace(p)
    mask = torch.full((w.B, w.H, w.T_m, w.T_n), -1.0, dtype=torch.float32, device="cuda")
    api.sla2_router_soft(p, q, k, rw, tau, mask, ws)
    torch.cuda.synchronize()
    return mask.cpu().numpy(), api.sla2_num_selected(p)


def oracle_soft(inp, b, h, k, tau):
    w = inp.workload
    Wq, Wk = inp.router_w[0].astype(np.float64), inp.router_w[1].astype(np.float64)
    R = O.router_scores(inp.values("q", b, h), O.smooth_k(inp.values("k", b, h)), Wq, Wk, w.block_q, w.block_kv)
    return O.soft_topk_rows(R, k, tau)


@pytest.mark.parametrize("w,tau", CASES, ids=lambda x: x.name if hasattr(x, "name") else str(x))
def test_soft_router_matches_oracle(w, tau):
    import torch
    from paper_2602_12675_amd import api
    inp = W.generate(w)
    got, k = run_soft(api, torch, inp, tau)
    assert k == w.k and 0 < k < w.T_n
    for b in range(w.B):
        for h in range(w.H):
            want = oracle_soft(inp, b, h, k, tau)
            np.testing.assert_allclose(got[b, h], want, rtol=0, atol=1e-6)
            np.testing.assert_allclose(got[b, h].astype(np.float64).sum(axis=1), k, rtol=0, atol=1e-4 * max(1, k))


@pytest.mark.parametrize("frac,value", [(0.0, 0.0), (1.0, 1.0)])
def test_soft_router_limits(frac, value):
    import torch
    from paper_2602_12675_amd import api
    inp = W.generate(W.TINY)
    got, k = run_soft(api, torch, inp, 0.1, topk_frac=frac)
    assert k in (0, W.TINY.T_n)
    assert np.all(got == value)


def test_soft_router_rejects_bad_tau():
    import torch
    from paper_2602_12675_amd import api
    w = W.TINY
    p = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac, dtype=api.SLA2_F32)
    ws = api.alloc_workspace(p)
    dummy = torch.zeros(16, device="cuda")
    for tau in (0.0, -1.0, float("nan")):
        assert api.sla2_router_soft(p, dummy, dummy, dummy, tau, dummy, ws, check=False) == api.SLA2_EINVAL
