"""GPU parity of the bf16 forward path (matrix-core kernels) against the oracle,
through the C ABI.  Tolerance for bf16 storage with fp32 accumulation: relative
L2 error of the output <= 2e-2 per head (the oracle works on the same bf16
input values in fp64 and is not rounded to bf16)."""
import numpy as np
import pytest

import sla2_oracle as O
from helpers import check_mask, oracle_heads, rel_l2, rows_ok, run_dense, run_forward
from paper_2602_12675_amd import workloads as W

pytestmark = pytest.mark.gpu

BF16_REL_L2 = 2e-2

BASE = W.TINY.replace(dtype="bf16", per_head_freq=True)
CASES = [
    BASE.replace(name="bf16-d128-bq128", grid=(5, 16, 33), d=128, block_q=128, H=3, topk_frac=0.1),     # N = 2640: 21 q blocks (tail 80), 42 kv blocks (tail 16)
    BASE.replace(name="bf16-d128-bq128-ragged", grid=(3, 11, 31), d=128, block_q=128, topk_frac=0.2),   # N = 1023: tails 127 / 63
    BASE.replace(name="bf16-d64-bq64", grid=(3, 11, 31), d=64, block_q=64, topk_frac=0.125),
    BASE.replace(name="bf16-d128-bq64", grid=(2, 13, 37), d=128, block_q=64, topk_frac=0.25),           # N = 962
    BASE.replace(name="bf16-d64-bq128", grid=(2, 13, 37), d=64, block_q=128, topk_frac=0.25),
    BASE.replace(name="bf16-one-block", grid=(1, 5, 8), d=128, block_q=128, topk_frac=0.5),             # N = 40
    BASE.replace(name="bf16-batch2", B=2, grid=(2, 8, 24), d=128, block_q=128, topk_frac=0.3),          # N = 384
]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_forward_bf16_matches_oracle(w):
    import torch
    from paper_2602_12675_amd import api
    inp = W.generate(w)
    r = run_forward(api, torch, inp)
    ref = oracle_heads(inp)
    L = api.sla2_workspace_layout(r["p"])
    BH = w.B * w.H
    h_total = api.workspace_view(r["ws"], L.h_total, torch.float32, (BH, w.d, w.d)).cpu().numpy()
    z_total = api.workspace_view(r["ws"], L.z_total, torch.float32, (BH, w.d)).cpu().numpy()
    k_mean = api.workspace_view(r["ws"], L.k_mean, torch.float64, (BH, w.d)).cpu().numpy()
    lnz = api.workspace_view(r["ws"], L.k_stats, torch.float32, (BH, w.N)).cpu().numpy()
    for (b, h), o in ref.items():
        bh = b * w.H + h
        assert check_mask(r["idx"][b, h], o["R"], o["sel"]) == 0
        np.testing.assert_allclose(k_mean[b * w.H + h], inp.values("k", b, h).mean(axis=0), rtol=1e-11, atol=1e-14)
        Ks = O.smooth_k(inp.values("k", b, h))
        ref_lnz = np.log(np.exp(Ks - Ks.max(axis=1, keepdims=True)).sum(axis=1)) + Ks.max(axis=1)
        np.testing.assert_allclose(lnz[bh], ref_lnz, rtol=0, atol=1e-4)
        hj, zj = O.kv_state(O.phi(Ks), inp.values("v", b, h), w.block_kv)
        assert rel_l2(h_total[bh], hj.sum(axis=0)) < 5e-3          # K^phi rounded to bf16 before the product
        assert rel_l2(z_total[bh], zj.sum(axis=0)) < 1e-4
        assert rel_l2(r["out"][b, h], o["O"]) <= BF16_REL_L2, (b, h, rel_l2(r["out"][b, h], o["O"]))
        rows_ok(r["out"][b, h], o["O"])
        fin = np.isfinite(o["L"])
        np.testing.assert_allclose(r["lse"][b, h][fin], o["L"][fin], rtol=0, atol=2e-2)
    assert not np.isnan(r["out"]).any()


def test_forward_bf16_branches_separately():
    """alpha = 1 isolates the sparse branch, alpha = 0 the linear branch: each
    must meet the tolerance on its own, not only their mix."""
    import torch
    from paper_2602_12675_amd import api
    w = CASES[0]
    inp = W.generate(w)
    for a, key in ((1.0, "O_s"), (0.0, "O_l")):
        al = np.full((w.H,), a, dtype=np.float32)
        r = run_forward(api, torch, inp, alpha=al)
        ref = oracle_heads(inp, alpha=al)
        for (b, h), o in ref.items():
            assert rel_l2(r["out"][b, h], o[key]) <= BF16_REL_L2, (key, h)
            rows_ok(r["out"][b, h], o[key])


@pytest.mark.parametrize("frac,alpha", [(0.0, 0.0), (1.0, 1.0), (0.0, 0.6), (1.0, 0.4)])
def test_forward_bf16_degenerate_branches(frac, alpha):
    import torch
    from paper_2602_12675_amd import api
    w = CASES[1].replace(name="deg", topk_frac=frac)
    inp = W.generate(w)
    al = np.full((w.H,), alpha, dtype=np.float32)
    r = run_forward(api, torch, inp, alpha=al)
    ref = oracle_heads(inp, alpha=al)
    for (b, h), o in ref.items():
        assert rel_l2(r["out"][b, h], o["O"]) <= BF16_REL_L2
        rows_ok(r["out"][b, h], o["O"])
    assert not np.isnan(r["out"]).any()


def test_forward_bf16_alpha_per_block_no_smoothing():
    import torch
    from paper_2602_12675_amd import api
    w = CASES[1]
    inp = W.generate(w)
    al = np.random.default_rng(5).uniform(size=(w.H, w.T_m)).astype(np.float32)
    r = run_forward(api, torch, inp, alpha=al, alpha_per_block=1, flags=api.SLA2_FLAG_NO_SMOOTH_K)
    ref = oracle_heads(inp, alpha=al, smooth=False)
    for (b, h), o in ref.items():
        assert check_mask(r["idx"][b, h], o["R"], o["sel"]) == 0
        assert rel_l2(r["out"][b, h], o["O"]) <= BF16_REL_L2
        rows_ok(r["out"][b, h], o["O"])


def test_forward_bf16_large_key_offset():
    """A large common offset on every key (what K-smoothing exists for): the
    mask and the sparse branch must not move, the output stays in tolerance."""
    import torch
    from paper_2602_12675_amd import api
    w = CASES[1]
    inp = W.generate(w)
    kv = W.bf16_bits_to_f32(inp.k) + np.float32(6.0)
    inp.k = W.f32_to_bf16_bits(kv)
    r = run_forward(api, torch, inp)
    ref = oracle_heads(inp)
    for (b, h), o in ref.items():
        assert check_mask(r["idx"][b, h], o["R"], o["sel"]) == 0
        assert rel_l2(r["out"][b, h], o["O"]) <= BF16_REL_L2
        rows_ok(r["out"][b, h], o["O"])


def test_forward_bf16_deterministic():
    import torch
    from paper_2602_12675_amd import api
    inp = W.generate(CASES[0])
    a = run_forward(api, torch, inp)
    b = run_forward(api, torch, inp)
    assert np.array_equal(a["out"], b["out"]) and np.array_equal(a["lse"], b["lse"])


DENSE_CASES = [CASES[0], CASES[1], BASE.replace(name="dense-d64", grid=(3, 11, 31), d=64, block_q=128),
               # the d = 128 kernel works on 256 query rows and on tiles of 64 keys through three buffers: lengths of one
               # row, less than a tile, one, two and three tiles with a tail, and a tail of one query row and one key
               BASE.replace(name="dense-N1", grid=(1, 1, 1), d=128, block_q=128, H=2),
               BASE.replace(name="dense-N50", grid=(1, 5, 10), d=128, block_q=128, H=2),
               BASE.replace(name="dense-N64", grid=(1, 8, 8), d=128, block_q=128, H=2),
               BASE.replace(name="dense-N130", grid=(1, 10, 13), d=128, block_q=128, H=2),
               BASE.replace(name="dense-N200", grid=(1, 10, 20), d=128, block_q=128, H=2),
               BASE.replace(name="dense-N769", grid=(1, 1, 769), d=128, block_q=128, B=2, H=3),
               BASE.replace(name="dense-N2049", grid=(1, 3, 683), d=128, block_q=128, H=2)] + [
    # around the 256-row workgroup and the three-buffer period
    BASE.replace(name="dense-N%d" % n, grid=(1, 1, n), d=128, block_q=128, H=2) for n in (191, 255, 256, 257, 385, 513)]


@pytest.mark.parametrize("w", DENSE_CASES, ids=lambda w: w.name)
def test_dense_baseline_matches_dense_attention(w):
    """The in-build comparator against the oracle with every block kept and
    alpha = 1 (= softmax(QK^T/sqrt d)V, pinned to the textbook routine)."""
    import torch
    from paper_2602_12675_amd import api
    inp = W.generate(w)
    out = run_dense(api, torch, inp)
    ref = oracle_heads(inp, alpha=np.ones((w.H,), np.float32), topk_frac=1.0)
    for (b, h), o in ref.items():
        assert rel_l2(out[b, h], o["O"]) <= BF16_REL_L2
        rows_ok(out[b, h], o["O"])
