"""GPU parity of the backward pass (Alg. 3 plus the chain through phi, the smoothing of K and the mix)
against the oracle, through the C ABI: sla2_forward with SLA2_FLAG_SAVE_FOR_BACKWARD, then sla2_backward
on the same workspace.  fp32 tensors: absolute tolerance; bf16 tensors: relative L2 (the gradients are
taken in fp32 from bf16 inputs and from the bf16 O^s, O^l the forward kept, and stored as bf16)."""
import numpy as np
import pytest

import sla2_oracle as O
from paper_2602_12675_amd import workloads as W

pytestmark = pytest.mark.gpu

BASE = W.TINY.replace(per_head_freq=True)
CASES = [
    (BASE.replace(name="bwd-f32-tiny"), False, True),
    (BASE.replace(name="bwd-f32-ragged", grid=(3, 11, 31), H=3), True, True),                               # N = 1023
    (BASE.replace(name="bwd-f32-d128-bq128", grid=(2, 13, 37), d=128, block_q=128, topk_frac=0.3), False, False),
    (BASE.replace(name="bwd-f32-b2", grid=(1, 9, 23), B=2, H=2, topk_frac=0.3), True, False),               # N = 207
    (BASE.replace(name="bwd-bf16-d128-bq128", grid=(5, 16, 33), d=128, block_q=128, H=2, dtype="bf16", topk_frac=0.1), False, True),
    (BASE.replace(name="bwd-bf16-ragged-bq64", grid=(3, 11, 31), d=128, block_q=64, dtype="bf16", topk_frac=0.2), True, True),
    (BASE.replace(name="bwd-bf16-fp8-forward", grid=(3, 11, 31), d=128, block_q=128, dtype="bf16", quant="fp8", topk_frac=0.2), False, True),
    (BASE.replace(name="bwd-bf16-d64", grid=(3, 11, 31), d=64, block_q=128, dtype="bf16", topk_frac=0.125), False, True),
    (BASE.replace(name="bwd-bf16-d64-bq64-b2", grid=(2, 13, 37), d=64, block_q=64, B=2, H=2, dtype="bf16", topk_frac=0.25), True, True),
    (BASE.replace(name="bwd-bf16-per-block-alpha-no-smooth", grid=(3, 11, 31), d=128, block_q=128, H=3, dtype="bf16", topk_frac=0.15), True, False),
    (BASE.replace(name="bwd-bf16-one-short-block", grid=(1, 5, 9), d=128, block_q=128, dtype="bf16", topk_frac=1.0), False, True),       # N = 45
    (BASE.replace(name="bwd-bf16-int8-forward", grid=(3, 11, 31), d=128, block_q=64, dtype="bf16", quant="int8", topk_frac=0.2), False, True),
    (BASE.replace(name="bwd-bf16-fp8v-forward", grid=(3, 11, 31), d=128, block_q=128, dtype="bf16", quant="fp8v", topk_frac=0.2), False, True),
]


def run_fwd_bwd(api, torch, inp, alpha, per_block, smooth, dout):
    w = inp.workload
    dt = api.SLA2_BF16 if w.dtype == "bf16" else api.SLA2_F32
    flags = api.SLA2_FLAG_SAVE_FOR_BACKWARD | (0 if smooth else api.SLA2_FLAG_NO_SMOOTH_K)
    p = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac, dtype=dt,
                        quant_mode=api.QUANT_MODES[w.quant], alpha_per_block=int(per_block), flags=flags)
    q, k, v = (api.to_device(a, dt) for a in (inp.q, inp.k, inp.v))
    rw = torch.from_numpy(inp.router_w).cuda()
    al = torch.from_numpy(np.ascontiguousarray(alpha, dtype=np.float32)).cuda()
    ws = api.alloc_workspace(p)
    kk = api.sla2_num_selected(p)
    out = torch.zeros_like(q)
    idx = torch.full((w.B, w.H, w.T_m, max(kk, 1)), -1, dtype=torch.int32, device="cuda")
    api.sla2_forward(p, q, k, v, rw, al, out, block_idx=idx, workspace=ws)
    go = api.to_device(dout, dt)
    dq, dk, dv = (torch.full_like(q, float("nan")) for _ in range(3))
    dal = torch.full_like(al, float("nan"))
    api.sla2_backward(p, q, k, v, al, go, dq, dk, dv, dal, ws)
    torch.cuda.synchronize()
    return dict(dq=dq.float().cpu().numpy(), dk=dk.float().cpu().numpy(), dv=dv.float().cpu().numpy(),
                dalpha=dal.cpu().numpy(), idx=idx.cpu().numpy()[..., :kk], go=go.float().cpu().numpy())


def rel(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b) / max(np.linalg.norm(b), 1e-30))


@pytest.mark.parametrize("w,per_block,smooth", CASES, ids=lambda x: x.name if hasattr(x, "name") else str(int(x)))
def test_backward_matches_oracle(w, per_block, smooth):
    import torch
    from paper_2602_12675_amd import api
    inp = W.generate(w)
    rng = np.random.default_rng(7)
    alpha = rng.uniform(0.1, 0.9, size=(w.H, w.T_m) if per_block else (w.H,)).astype(np.float32)
    dout = rng.normal(size=(w.B, w.H, w.N, w.d)).astype(np.float32)
    if w.dtype == "bf16":
        dout = W.f32_to_bf16_bits(dout)
    r = run_fwd_bwd(api, torch, inp, alpha, per_block, smooth, dout)
    dal_ref = np.zeros(alpha.shape, dtype=np.float64)
    tol = 2e-2 if w.dtype == "bf16" else None
    for b in range(w.B):
        for h in range(w.H):
            Q, K, V = (inp.values(n, b, h) for n in ("q", "k", "v"))
            g = O.backward_head(Q, K, V, r["idx"][b, h], alpha[h].astype(np.float64), r["go"][b, h].astype(np.float64),
                                w.block_q, w.block_kv, smooth=smooth,
                                quant={"none": O.QUANT_NONE, "fp8": O.QUANT_FP8, "int8": O.QUANT_INT8, "fp8v": O.QUANT_FP8_V}[w.quant])
            dal_ref[h] += g["dalpha"] if per_block else g["dalpha"].sum()
            for name in ("dq", "dk", "dv"):
                want = g["d" + name[1].upper()]
                if tol is None:
                    np.testing.assert_allclose(r[name][b, h], want, rtol=0, atol=2e-4 * max(1.0, np.abs(want).max()),
                                               err_msg="%s b%d h%d" % (name, b, h))
                else:
                    assert rel(r[name][b, h], want) <= tol, (name, b, h, rel(r[name][b, h], want))
    if tol is None:
        np.testing.assert_allclose(r["dalpha"], dal_ref, rtol=1e-4, atol=1e-3)
    else:
        np.testing.assert_allclose(r["dalpha"], dal_ref, rtol=3e-2, atol=3e-2 * np.abs(dal_ref).max())
    assert all(np.isfinite(r[n]).all() for n in ("dq", "dk", "dv", "dalpha"))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("frac", [0.0, 1.0])
def test_backward_with_an_empty_branch(frac, dtype):
    import torch
    from paper_2602_12675_amd import api
    w = BASE.replace(name="bwd-empty-%g-%s" % (frac, dtype), grid=(3, 11, 31), topk_frac=frac)
    if dtype == "bf16":
        w = w.replace(d=128, block_q=128, dtype="bf16")
    inp = W.generate(w)
    rng = np.random.default_rng(8)
    alpha = rng.uniform(0.1, 0.9, size=(w.H,)).astype(np.float32)
    dout = rng.normal(size=(w.B, w.H, w.N, w.d)).astype(np.float32)
    if dtype == "bf16":
        dout = W.f32_to_bf16_bits(dout)
    r = run_fwd_bwd(api, torch, inp, alpha, False, True, dout)
    assert all(np.isfinite(r[n]).all() for n in ("dq", "dk", "dv", "dalpha"))
    for h in range(w.H):
        Q, K, V = (inp.values(n, 0, h) for n in ("q", "k", "v"))
        g = O.backward_head(Q, K, V, r["idx"][0, h], float(alpha[h]), r["go"][0, h].astype(np.float64), w.block_q, w.block_kv)
        for name in ("dq", "dk", "dv"):
            want = g["d" + name[1].upper()]
            if dtype == "f32":
                np.testing.assert_allclose(r[name][0, h], want, rtol=0, atol=2e-4 * max(1.0, np.abs(want).max()))
            else:
                assert rel(r[name][0, h], want) <= 2e-2, (name, h, rel(r[name][0, h], want))
        if dtype == "f32":
            np.testing.assert_allclose(r["dalpha"][h], g["dalpha"].sum(), rtol=1e-4, atol=1e-3)
        else:
            np.testing.assert_allclose(r["dalpha"][h], g["dalpha"].sum(), rtol=3e-2, atol=3e-2 * abs(g["dalpha"].sum()))


def test_backward_needs_the_save_flag():
    import torch
    from paper_2602_12675_amd import api
    w = BASE
    p = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac, dtype=api.SLA2_F32)
    ws = api.alloc_workspace(p)
    t = torch.zeros(64, device="cuda")
    assert api.sla2_backward(p, t, t, t, t, t, t, t, t, t, ws, check=False) == api.SLA2_EINVAL


@pytest.mark.parametrize("w", [
    BASE.replace(name="bwd-strided-f32", grid=(3, 11, 31), H=3),
    BASE.replace(name="bwd-strided-bf16", grid=(3, 11, 31), d=128, block_q=128, B=2, H=2, dtype="bf16", topk_frac=0.2),
], ids=lambda w: w.name)
def test_backward_strided_equals_contiguous(w):
    """q, k, v as slices of a packed [B, N, 3, H, d] projection, dout as [B, N, H, d], and the gradients
    written into the slices of a packed [B, N, 3, H, d + pad] buffer: the same bits as the contiguous
    call, and nothing written between the rows."""
    import torch
    from paper_2602_12675_amd import api
    inp = W.generate(w)
    rng = np.random.default_rng(9)
    alpha = rng.uniform(0.1, 0.9, size=(w.H,)).astype(np.float32)
    dout = rng.normal(size=(w.B, w.H, w.N, w.d)).astype(np.float32)
    if w.dtype == "bf16":
        dout = W.f32_to_bf16_bits(dout)
    ref = run_fwd_bwd(api, torch, inp, alpha, False, True, dout)
    dt = api.SLA2_BF16 if w.dtype == "bf16" else api.SLA2_F32
    q, k, v = (api.to_device(a, dt) for a in (inp.q, inp.k, inp.v))
    pad = 8
    qkv = torch.empty((w.B, w.N, 3, w.H, w.d + pad), dtype=q.dtype, device="cuda")
    grads = torch.full_like(qkv, 7.0)
    for x, t in enumerate((q, k, v)):
        qkv[:, :, x, :, :w.d] = t.permute(0, 2, 1, 3)
    go = api.to_device(dout, dt).permute(0, 2, 1, 3).contiguous()                  # [B, N, H, d]
    row = 3 * w.H * (w.d + pad)
    in_stride = (w.N * row, w.d + pad, row)
    out_stride = (w.N * w.H * w.d, w.d, w.H * w.d)
    p = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac, dtype=dt,
                        flags=api.SLA2_FLAG_SAVE_FOR_BACKWARD, in_stride=in_stride, out_stride=out_stride)
    rw = torch.from_numpy(inp.router_w).cuda()
    al = torch.from_numpy(alpha).cuda()
    ws = api.alloc_workspace(p)
    out = torch.empty((w.B, w.N, w.H, w.d), dtype=q.dtype, device="cuda")
    api.sla2_forward(p, qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], rw, al, out, workspace=ws)
    dal = torch.empty_like(al)
    api.sla2_backward(p, qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], al, go, grads[:, :, 0], grads[:, :, 1], grads[:, :, 2],
                      dal, ws)
    torch.cuda.synchronize()
    gr = grads.float().cpu().numpy()
    assert np.all(gr[..., w.d:] == 7.0)
    for x, name in enumerate(("dq", "dk", "dv")):
        assert np.array_equal(gr[:, :, x, :, :w.d].transpose(0, 2, 1, 3), ref[name]), name
    assert np.array_equal(dal.cpu().numpy(), ref["dalpha"])
