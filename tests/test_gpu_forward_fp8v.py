"""GPU parity of the low-bit mode that also quantises V for the second product (Alg. 2 as
printed: quant(P) quant(V_j); Sec. 5) against the oracle's step-by-step statement, through
the C ABI.  Byte work (e4m3 codes and scales of K and of V, the latter through the token
order of the stored tile) is compared bit for bit; the output within relative L2 5e-2 per
head (the low-bit tolerance)."""
import numpy as np
import pytest

import sla2_oracle as O
from helpers import check_mask, oracle_heads, rel_l2, rows_ok, run_forward
from paper_2602_12675_amd import workloads as W
from test_gpu_forward_fp8 import e4m3_decode

pytestmark = pytest.mark.gpu

LOWBIT_REL_L2 = 5e-2

BASE = W.TINY.replace(dtype="bf16", quant="fp8v", per_head_freq=True)
CASES = [
    BASE.replace(name="fp8v-d128-bq128", grid=(5, 16, 33), d=128, block_q=128, H=3, topk_frac=0.1),      # N = 2640
    BASE.replace(name="fp8v-d128-bq128-ragged", grid=(3, 11, 31), d=128, block_q=128, topk_frac=0.2),    # N = 1023
    BASE.replace(name="fp8v-d64-bq64", grid=(3, 11, 31), d=64, block_q=64, topk_frac=0.125),
    BASE.replace(name="fp8v-d128-bq64", grid=(2, 13, 37), d=128, block_q=64, topk_frac=0.25),
    BASE.replace(name="fp8v-d64-bq128", grid=(2, 13, 37), d=64, block_q=128, topk_frac=0.25),
    BASE.replace(name="fp8v-one-block", grid=(1, 5, 8), d=128, block_q=128, topk_frac=0.5),
]

# byte 32 g + b of a row of the stored V-code tile holds this token of the key block (sla2.h, v_fp8)
TOKEN_OF_BYTE = np.array([32 * (b // 16) + 8 * ((b % 16) // 4) + 4 * g + b % 4 for g in range(2) for b in range(32)])


def test_token_order_is_a_permutation():
    assert sorted(TOKEN_OF_BYTE.tolist()) == list(range(64))


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_forward_fp8v_matches_oracle(w):
    import torch
    from paper_2602_12675_amd import api
    inp = W.generate(w)
    r = run_forward(api, torch, inp)
    ref = oracle_heads(inp)
    L = api.sla2_workspace_layout(r["p"])
    BH = w.B * w.H
    vcodes = api.workspace_view(r["ws"], L.v_fp8, torch.uint8, (BH, w.T_n, w.d, w.block_kv)).cpu().numpy()
    vscales = api.workspace_view(r["ws"], L.v_scale, torch.float32, (BH, w.T_n)).cpu().numpy()
    kscales = api.workspace_view(r["ws"], L.k_scale, torch.float32, (BH, w.T_n)).cpu().numpy()
    worst = 0.0
    for (b, h), o in ref.items():
        bh = b * w.H + h
        assert check_mask(r["idx"][b, h], o["R"], o["sel"]) == 0
        V32 = inp.values("v", b, h).astype(np.float32)
        K32 = O.smooth_k_f32(inp.values("k", b, h))
        mism = 0
        for j in range(w.T_n):
            c0, c1 = j * w.block_kv, min(w.N, (j + 1) * w.block_kv)
            vals, s = O.quant_block_e4m3(V32[c0:c1])                    # [tokens, d]
            assert vscales[bh, j] == s
            assert kscales[bh, j] == O.quant_block_e4m3(K32[c0:c1])[1]
            tile = e4m3_decode(vcodes[bh, j])                           # [d, 64 bytes]
            by_token = np.zeros((w.block_kv, w.d))
            by_token[TOKEN_OF_BYTE] = tile.T                            # row = token, column = channel
            mism += int((by_token[:c1 - c0] != vals).sum())
            assert not by_token[c1 - c0:].any()                         # tokens past the end are zero
        assert mism == 0
        e = rel_l2(r["out"][b, h], o["O"])
        rows_ok(r["out"][b, h], o["O"], "fp8v")
        worst = max(worst, e)
        assert e <= LOWBIT_REL_L2, (b, h, e)
        fin = np.isfinite(o["L"])
        np.testing.assert_allclose(r["lse"][b, h][fin], o["L"][fin], rtol=0, atol=2e-2)
    assert not np.isnan(r["out"]).any()
    print("worst rel-L2 vs the oracle: %.4f" % worst)


def test_forward_fp8v_sparse_branch_alone_sees_the_rounded_v():
    """alpha = 1: the low-bit branch on its own.  The kernel must sit closer to the oracle of this
    mode than that oracle sits to the FP8 mode with V left alone - i.e. it reproduces the rounding
    of V, not just the attention."""
    import torch
    from paper_2602_12675_amd import api
    w = CASES[0]
    inp = W.generate(w)
    al = np.ones((w.H,), np.float32)
    r = run_forward(api, torch, inp, alpha=al)
    lo = oracle_heads(inp, alpha=al)
    f8 = oracle_heads(inp, alpha=al, quant=O.QUANT_FP8)
    for key in lo:
        b, h = key
        e_kernel = rel_l2(r["out"][b, h], lo[key]["O"])
        rows_ok(r["out"][b, h], lo[key]["O"], "fp8v")
        e_v = rel_l2(lo[key]["O"], f8[key]["O"])
        assert e_kernel <= LOWBIT_REL_L2
        assert e_kernel < 0.5 * e_v, (e_kernel, e_v)


@pytest.mark.parametrize("frac,alpha", [(0.0, 0.3), (1.0, 1.0)])
def test_forward_fp8v_degenerate(frac, alpha):
    import torch
    from paper_2602_12675_amd import api
    w = CASES[1].replace(name="deg", topk_frac=frac)
    inp = W.generate(w)
    al = np.full((w.H,), alpha, dtype=np.float32)
    r = run_forward(api, torch, inp, alpha=al)
    ref = oracle_heads(inp, alpha=al)
    for (b, h), o in ref.items():
        assert rel_l2(r["out"][b, h], o["O"]) <= LOWBIT_REL_L2
        rows_ok(r["out"][b, h], o["O"], "fp8v")
    assert not np.isnan(r["out"]).any()


def test_forward_fp8v_blocks_of_very_different_v_scale():
    """The running output is carried in units of the current block's V scale; blocks whose V differ by
    orders of magnitude exercise the hand-over between units."""
    import torch
    from paper_2602_12675_amd import api
    w = CASES[1]
    inp = W.generate(w)
    vals = W.bf16_bits_to_f32(inp.v)
    for j in range(w.T_n):
        vals[:, :, j * w.block_kv:(j + 1) * w.block_kv] *= np.float32(4.0 ** ((j % 7) - 3))
    inp.v[...] = W.f32_to_bf16_bits(vals)
    r = run_forward(api, torch, inp)
    ref = oracle_heads(inp)
    for (b, h), o in ref.items():
        assert rel_l2(r["out"][b, h], o["O"]) <= LOWBIT_REL_L2
        rows_ok(r["out"][b, h], o["O"], "fp8v")
    assert not np.isnan(r["out"]).any()
