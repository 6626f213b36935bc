"""GPU parity of the router (pooling, colmean, projections, scores, top-k)
against the oracle, through the C ABI."""
import numpy as np
import pytest

import sla2_oracle as O
from helpers import check_mask
from paper_2602_12675_amd import workloads as W

pytestmark = pytest.mark.gpu


def run_router(api, torch, inp, flags=0):
    w = inp.workload
    dt = api.SLA2_BF16 if w.dtype == "bf16" else api.SLA2_F32
    p = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac, dtype=dt, flags=flags)
    q, k = api.to_device(inp.q, dt), api.to_device(inp.k, dt)
    rw = torch.from_numpy(inp.router_w).cuda()
    ws = api.alloc_workspace(p)
    kk = api.sla2_num_selected(p)
    idx = torch.full((w.B, w.H, w.T_m, max(kk, 1)), -1, dtype=torch.int32, device="cuda")
    api.sla2_router(p, q, k, rw, idx, ws)
    torch.cuda.synchronize()
    return p, ws, idx.cpu().numpy()[..., :kk], kk


CASES = [
    W.TINY,
    W.TINY.replace(name="tiny-ragged", grid=(3, 11, 31)),                                   # N = 1023
    W.TINY.replace(name="f32-d128", grid=(2, 13, 37), d=128, block_q=128, topk_frac=0.3),    # N = 962
    W.TINY.replace(name="bf16-d128", grid=(5, 16, 33), d=128, block_q=128, dtype="bf16", H=3,
                   topk_frac=0.1, per_head_freq=True),                                      # N = 2640
    W.TINY.replace(name="bf16-d64-wide", grid=(9, 30, 52), d=64, dtype="bf16", H=1, topk_frac=0.05),  # T_n = 220
    W.TINY.replace(name="bf16-d64-700-blocks", grid=(16, 50, 56), d=64, dtype="bf16", H=1, topk_frac=0.03),    # N = 44800, T_n = 700
    W.TINY.replace(name="bf16-d128-1200-blocks", grid=(24, 50, 64), d=128, block_q=128, dtype="bf16", H=1,
                   topk_frac=0.15, extra_tokens=3),                                                        # N = 76803, T_n = 1201
    W.TINY.replace(name="bf16-d64-2048-blocks", grid=(32, 64, 64), d=64, dtype="bf16", H=1, topk_frac=0.01),  # T_n = 2048 (the limit)
]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_router_matches_oracle(w):
    import torch
    from paper_2602_12675_amd import api
    inp = W.generate(w)
    p, ws, idx, kk = run_router(api, torch, inp)
    assert kk == w.k
    L = api.sla2_workspace_layout(p)
    BH = w.B * w.H
    q_sum = api.workspace_view(ws, L.q_sum, torch.float64, (BH, w.T_m, w.d)).cpu().numpy()
    k_sum = api.workspace_view(ws, L.k_sum, torch.float64, (BH, w.T_n, w.d)).cpu().numpy()
    Wq, Wk = inp.router_w[0].astype(np.float64), inp.router_w[1].astype(np.float64)
    diff_rows = 0
    for b in range(w.B):
        for h in range(w.H):
            Q, K = inp.values("q", b, h), inp.values("k", b, h)
            bh = b * w.H + h
            # pooled sums and the column mean: same numbers up to summation order
            cnt_q = np.minimum(w.block_q, w.N - np.arange(w.T_m) * w.block_q)[:, None]
            cnt_k = np.minimum(w.block_kv, w.N - np.arange(w.T_n) * w.block_kv)[:, None]
            np.testing.assert_allclose(q_sum[bh] / cnt_q, O.pool(Q, w.block_q), rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(k_sum[bh] / cnt_k, O.pool(K, w.block_kv), rtol=1e-12, atol=1e-13)
            R = O.router_scores(Q, O.smooth_k(K), Wq, Wk, w.block_q, w.block_kv)
            sel = O.topk_rows(R, kk)
            diff_rows += check_mask(idx[b, h], R, sel)
    assert diff_rows == 0      # no exact ties in random data: the lists are identical


def test_router_ties_break_toward_lower_index():
    """Equal keys everywhere (K constant over tokens): every score of a row is
    the same number, so the k lowest indices must be kept."""
    import torch
    from paper_2602_12675_amd import api
    w = W.TINY.replace(name="ties", topk_frac=0.25)
    inp = W.generate(w)
    inp.k[:] = inp.k[:, :, :1, :]
    _, _, idx, kk = run_router(api, torch, inp, flags=api.SLA2_FLAG_NO_SMOOTH_K)
    assert kk == 4
    assert np.array_equal(idx, np.broadcast_to(np.arange(4, dtype=np.int32), idx.shape))


def test_router_duplicate_blocks_tie_window():
    """Two key blocks with identical tokens have identical scores; whichever
    the top-k boundary falls on, the lower index wins (oracle rule)."""
    import torch
    from paper_2602_12675_amd import api
    w = W.TINY.replace(name="dups", topk_frac=0.25)
    inp = W.generate(w)
    for j in range(0, 16, 2):
        inp.k[:, :, (j + 1) * 64:(j + 2) * 64] = inp.k[:, :, j * 64:(j + 1) * 64]
    p, ws, idx, kk = run_router(api, torch, inp)
    Wq, Wk = inp.router_w[0].astype(np.float64), inp.router_w[1].astype(np.float64)
    for h in range(w.H):
        Q, K = inp.values("q", 0, h), inp.values("k", 0, h)
        R = O.router_scores(Q, O.smooth_k(K), Wq, Wk, 64, 64)
        check_mask(idx[0, h], R, O.topk_rows(R, kk))


@pytest.mark.parametrize("frac", [0.0, 1.0])
def test_router_degenerate_k(frac):
    import torch
    from paper_2602_12675_amd import api
    w = W.TINY.replace(name="deg", topk_frac=frac)
    inp = W.generate(w)
    _, _, idx, kk = run_router(api, torch, inp)
    assert kk == (0 if frac == 0.0 else w.T_n)
    if kk:
        assert np.array_equal(idx, np.broadcast_to(np.arange(kk, dtype=np.int32), idx.shape))


def test_router_identity_weights_is_topk_of_pooled_scores():
    """router_w = (I, I): the learnable router reduces to Top-k of pool(Q) pool(K)^T, the fixed
    router the paper ablates against (Sec. 9.4, "Topk-router")."""
    import torch
    from paper_2602_12675_amd import api
    w = W.TINY.replace(name="identity-router", grid=(5, 16, 33), d=128, block_q=128, dtype="bf16", H=2,
                       topk_frac=0.1, per_head_freq=True)
    inp = W.generate(w)
    inp.router_w[:] = np.eye(w.d, dtype=np.float32)[None]
    _, _, idx, kk = run_router(api, torch, inp)
    for h in range(w.H):
        Q, K = inp.values("q", 0, h), inp.values("k", 0, h)
        R = O.pool(Q, w.block_q) @ O.pool(O.smooth_k(K), w.block_kv).T      # no projection, no scale
        assert check_mask(idx[0, h], R, O.topk_rows(R, kk)) == 0


def test_router_per_head_weights():
    """router_w_per_head = 1: one (Wq, Wk) pair per head, [H, 2, d, d]."""
    import torch
    from paper_2602_12675_amd import api
    w = W.TINY.replace(name="per-head-router", grid=(3, 11, 31), H=3, topk_frac=0.2)
    inp = W.generate(w)
    rng = np.random.default_rng(5)
    rw = (rng.normal(size=(w.H, 2, w.d, w.d)) / np.sqrt(w.d)).astype(np.float32)
    p = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac, dtype=api.SLA2_F32,
                        router_w_per_head=1)
    q, k = api.to_device(inp.q, api.SLA2_F32), api.to_device(inp.k, api.SLA2_F32)
    ws = api.alloc_workspace(p)
    kk = api.sla2_num_selected(p)
    idx = torch.full((w.B, w.H, w.T_m, kk), -1, dtype=torch.int32, device="cuda")
    api.sla2_router(p, q, k, torch.from_numpy(rw).cuda(), idx, ws)
    torch.cuda.synchronize()
    idx = idx.cpu().numpy()
    for h in range(w.H):
        Q, K = inp.values("q", 0, h), inp.values("k", 0, h)
        R = O.router_scores(Q, O.smooth_k(K), rw[h, 0].astype(np.float64), rw[h, 1].astype(np.float64), w.block_q, w.block_kv)
        assert check_mask(idx[0, h], R, O.topk_rows(R, kk)) == 0
