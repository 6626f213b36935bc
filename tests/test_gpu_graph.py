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


def test_forward_and_backward_under_graph_capture_replay_exactly():
    """The training pair - sla2_forward keeping its intermediates, then sla2_backward - captured into one
    graph: every replay reproduces the eager gradients bit for bit (the backward pass has no atomics and
    no data-dependent summation order), with the workspace scribbled over in between."""
    import torch
    from paper_2602_12675_amd import api
    w = W.TINY.replace(name="graph-bwd", grid=(5, 16, 33), d=128, block_q=128, H=3, dtype="bf16", quant="fp8",
                       topk_frac=0.1, per_head_freq=True)
    inp = W.generate(w)
    dt = api.SLA2_BF16
    p = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac, dtype=dt, quant_mode=api.QUANT_MODES["fp8"],
                        flags=api.SLA2_FLAG_SAVE_FOR_BACKWARD)
    q, k, v = (api.to_device(a, dt) for a in (inp.q, inp.k, inp.v))
    go = api.to_device(W.f32_to_bf16_bits(np.random.default_rng(3).normal(size=inp.q.shape).astype(np.float32)), dt)
    rw = torch.from_numpy(inp.router_w).cuda()
    al = torch.from_numpy(inp.alpha).cuda()
    ws = api.alloc_workspace(p)
    out = torch.zeros_like(q)
    dq, dk, dv = (torch.zeros_like(q) for _ in range(3))
    dal = torch.zeros_like(al)

    def both(stream=None):
        api.sla2_forward(p, q, k, v, rw, al, out, workspace=ws, stream=stream)
        api.sla2_backward(p, q, k, v, al, go, dq, dk, dv, dal, ws, stream=stream)

    both()
    torch.cuda.synchronize()
    ref = [t.clone() for t in (out, dq, dk, dv, dal)]
    both()                                              # eager, a second time: the same bits
    torch.cuda.synchronize()
    for t, r in zip((out, dq, dk, dv, dal), ref):
        assert torch.equal(t, r)

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            both(stream=side)
    torch.cuda.synchronize()
    scratch = torch.empty(1 << 20, device="cuda")
    for rep in range(3):
        for t in (out, dq, dk, dv, dal):
            t.zero_()
        ws.random_(0, 255)
        scratch.normal_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, r in zip((out, dq, dk, dv, dal), ref):
            assert torch.equal(t, r), rep
