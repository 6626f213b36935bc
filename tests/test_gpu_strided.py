"""q, k, v as the three slices of one packed [B, N, 3, H, d] projection and out as [B, N, H, d], passed
by strides: the result must be the contiguous call's result bit for bit (same arithmetic, other
addresses), in every precision mode, including ragged shapes; memory around the output rows must be
left alone."""
import numpy as np
import pytest

from helpers import oracle_heads, rel_l2, rows_ok, run_forward
from paper_2602_12675_amd import workloads as W

pytestmark = pytest.mark.gpu

BASE = W.TINY.replace(per_head_freq=True)
CASES = [
    BASE.replace(name="strided-f32", grid=(3, 11, 31), H=3),                                                   # N = 1023
    BASE.replace(name="strided-bf16", grid=(5, 16, 33), d=128, block_q=128, H=3, dtype="bf16", topk_frac=0.1),
    BASE.replace(name="strided-bf16-ragged-b2", grid=(3, 11, 31), d=128, block_q=128, B=2, H=2, dtype="bf16", topk_frac=0.2),
    BASE.replace(name="strided-fp8", grid=(3, 11, 31), d=128, block_q=128, H=2, dtype="bf16", quant="fp8", topk_frac=0.2),
    BASE.replace(name="strided-int8-d64", grid=(3, 11, 31), d=64, block_q=64, H=2, dtype="bf16", quant="int8", topk_frac=0.125),
    BASE.replace(name="strided-fp8v-bq64", grid=(2, 13, 37), d=128, block_q=64, H=2, dtype="bf16", quant="fp8v", topk_frac=0.25),
]


def run_strided(api, torch, inp):
    w = inp.workload
    dt = api.SLA2_BF16 if w.dtype == "bf16" else api.SLA2_F32
    q, k, v = (api.to_device(a, dt) for a in (inp.q, inp.k, inp.v))              # [B, H, N, d]
    qkv = torch.empty((w.B, w.N, 3, w.H, w.d), dtype=q.dtype, device="cuda")
    for x, t in enumerate((q, k, v)):
        qkv[:, :, x] = t.permute(0, 2, 1, 3)
    in_stride = (w.N * 3 * w.H * w.d, w.d, 3 * w.H * w.d)                        # batch, head, token
    # out: [B, N, H, d + pad] rows with a guard band after every head row
    pad = 8
    out = torch.full((w.B, w.N, w.H, w.d + pad), 7.0, dtype=q.dtype, device="cuda")
    out_stride = (w.N * w.H * (w.d + pad), w.d + pad, w.H * (w.d + pad))
    p = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac, dtype=dt,
                        quant_mode=api.QUANT_MODES[w.quant], in_stride=in_stride, out_stride=out_stride)
    rw = torch.from_numpy(inp.router_w).cuda()
    al = torch.from_numpy(np.ascontiguousarray(inp.alpha, dtype=np.float32)).cuda()
    ws = api.alloc_workspace(p)
    kk = api.sla2_num_selected(p)
    idx = torch.full((w.B, w.H, w.T_m, max(kk, 1)), -1, dtype=torch.int32, device="cuda")
    api.sla2_forward(p, qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], rw, al, out, block_idx=idx, workspace=ws)
    torch.cuda.synchronize()
    o = out.float().cpu().numpy()
    return o[..., :w.d].transpose(0, 2, 1, 3), o[..., w.d:], idx.cpu().numpy()[..., :kk]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_strided_call_equals_contiguous_call(w):
    import torch
    from paper_2602_12675_amd import api
    inp = W.generate(w)
    ref = run_forward(api, torch, inp, want_lse=False)
    got, guard, idx = run_strided(api, torch, inp)
    assert np.array_equal(idx, ref["idx"])
    assert np.array_equal(got, ref["out"])                 # bit for bit
    assert np.all(guard == 7.0)                            # nothing written between the rows
    o = oracle_heads(inp, heads=[(0, 0)])[(0, 0)]
    assert rel_l2(got[0, 0], o["O"]) <= (5e-2 if w.quant != "none" else 2e-2)
    rows_ok(got[0, 0], o["O"], w.quant)


def test_strided_router_and_dense():
    import torch
    from paper_2602_12675_amd import api
    w = CASES[1]
    inp = W.generate(w)
    dt = api.SLA2_BF16
    q, k, v = (api.to_device(a, dt) for a in (inp.q, inp.k, inp.v))
    qkv = torch.empty((w.B, w.N, 3, w.H, w.d), dtype=q.dtype, device="cuda")
    for x, t in enumerate((q, k, v)):
        qkv[:, :, x] = t.permute(0, 2, 1, 3)
    st = (w.N * 3 * w.H * w.d, w.d, 3 * w.H * w.d)
    ost = (w.N * w.H * w.d, w.d, w.H * w.d)
    rw = torch.from_numpy(inp.router_w).cuda()
    ps = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac, dtype=dt, in_stride=st, out_stride=ost)
    pc = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac, dtype=dt)
    kk = api.sla2_num_selected(pc)
    res = []
    for p, (a, b) in ((ps, (qkv[:, :, 0], qkv[:, :, 1])), (pc, (q, k))):
        ws = api.alloc_workspace(p)
        idx = torch.full((w.B, w.H, w.T_m, kk), -1, dtype=torch.int32, device="cuda")
        api.sla2_router(p, a, b, rw, idx, ws)
        mask = torch.empty((w.B, w.H, w.T_m, w.T_n), dtype=torch.float32, device="cuda")
        api.sla2_router_soft(p, a, b, rw, 0.1, mask, ws)
        torch.cuda.synchronize()
        res.append((idx.cpu().numpy(), mask.cpu().numpy()))
    assert np.array_equal(res[0][0], res[1][0]) and np.array_equal(res[0][1], res[1][1])
    od_s = torch.zeros((w.B, w.N, w.H, w.d), dtype=q.dtype, device="cuda")
    od_c = torch.zeros_like(q)
    api.sla2_dense_forward(ps, qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], od_s)
    api.sla2_dense_forward(pc, q, k, v, od_c)
    torch.cuda.synchronize()
    assert torch.equal(od_s.permute(0, 2, 1, 3), od_c)
