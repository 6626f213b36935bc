"""sla2_forward enqueues kernels only (no allocation, no synchronisation, no host reads), so a caller may
capture it into a HIP graph.  Every replay, with eager work and synchronisations of the program's own in
between, must reproduce the eager result bit for bit."""
import numpy as np
import pytest

from paper_2602_12675_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("quant", ["none", "fp8"])
def test_forward_under_graph_capture_replays_exactly(quant):
    import torch
    from paper_2602_12675_amd import api
    w = W.TINY.replace(name="graph-" + quant, grid=(5, 16, 33), d=128, block_q=128, H=3, dtype="bf16", quant=quant,
                       topk_frac=0.1, per_head_freq=True)
    inp = W.generate(w)
    dt = api.SLA2_BF16
    p = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac, dtype=dt, quant_mode=api.QUANT_MODES[quant])
    q, k, v = (api.to_device(a, dt) for a in (inp.q, inp.k, inp.v))
    rw = torch.from_numpy(inp.router_w).cuda()
    al = torch.from_numpy(inp.alpha).cuda()
    ws = api.alloc_workspace(p)
    out = torch.zeros_like(q)
    kk = api.sla2_num_selected(p)
    idx = torch.zeros((w.B, w.H, w.T_m, kk), dtype=torch.int32, device="cuda")
    lse = torch.zeros((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
    api.sla2_forward(p, q, k, v, rw, al, out, block_idx=idx, lse=lse, workspace=ws)      # eager reference (also warms up)
    torch.cuda.synchronize()
    ref_out, ref_idx, ref_lse = out.clone(), idx.clone(), lse.clone()

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            api.sla2_forward(p, q, k, v, rw, al, out, block_idx=idx, lse=lse, workspace=ws, stream=side)
    torch.cuda.synchronize()
    scratch = torch.empty(1 << 20, device="cuda")
    for rep in range(4):
        out.zero_(); idx.zero_(); lse.zero_()
        ws.random_(0, 255)                              # the workspace carries nothing from call to call
        scratch.normal_()                               # eager work of the program's own between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out), rep
        assert torch.equal(idx, ref_idx), rep
        assert torch.equal(lse, ref_lse), rep
