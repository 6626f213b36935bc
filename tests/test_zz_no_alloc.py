"""The router entry point that allocates nothing (sla2_router_static) against sla2_router, through the
C ABI: two calls in a row on one GPU, the second with a smaller input, so that whatever the first call
left in the library's device array must not leak into the second."""
import numpy as np
import pytest

from paper_2602_12675_amd import workloads as W



def _both(api, torch, w):
    inp = W.generate(w)
    dt = api.SLA2_BF16 if w.dtype == "bf16" else api.SLA2_F32
    p = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac, dtype=dt)
    q, k = (api.to_device(a, dt) for a in (inp.q, inp.k))
    rw = torch.from_numpy(inp.router_w).cuda()
    kk = api.sla2_num_selected(p)
    ref = torch.full((w.B, w.H, w.T_m, kk), -1, dtype=torch.int32, device="cuda")
    got = torch.full((w.B, w.H, w.T_m, kk), -2, dtype=torch.int32, device="cuda")
    ws = api.alloc_workspace(p)
    api.sla2_router(p, q, k, rw, ref, ws)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    api.sla2_router_static(p, q, k, rw, got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return ref.cpu().numpy(), got.cpu().numpy()


@pytest.mark.gpu
def test_static_router_matches_router_on_two_calls_in_a_row():
    import torch
    from paper_2602_12675_amd import api
    big = W.TINY.replace(name="static-a", dtype="bf16", B=1, H=3, d=128, block_q=128, grid=(5, 19, 37),
                         topk_frac=0.1, per_head_freq=True)             # N = 3515: ragged query and key blocks
    small = W.TINY.replace(name="static-b", dtype="f32", B=2, H=2, d=64, block_q=64, grid=(2, 9, 23),
                           topk_frac=0.25, per_head_freq=True)          # N = 414, other d, other element type
    for w in (big, small):
        ref, got = _both(api, torch, w)
        assert ref.min() >= 0
        np.testing.assert_array_equal(got, ref)                         # index work: bit-exact


def test_static_router_refuses_what_does_not_fit():
    from paper_2602_12675_amd import api
    p = api.make_params(1, 40, 75600, 128, 128, 64, 0.03)               # router arrays: 73 MB
    assert api.sla2_workspace_layout(p).block_idx > api.SLA2_STATIC_SCRATCH_BYTES
    assert api.sla2_router_static(p, 256, 256, 256, 256, check=False) == api.SLA2_EWORKSPACE
    p = api.make_params(1, 12, 32760, 128, 128, 64, 0.03)
    assert api.sla2_workspace_layout(p).block_idx <= api.SLA2_STATIC_SCRATCH_BYTES
