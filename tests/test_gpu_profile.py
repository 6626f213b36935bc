"""Per-stage event timing of the C ABI (sla2_profile_begin / _begin_sampled / _end): launch counts
per stage, sampling stride, argument checks.  Timing values are only required to be positive."""
import numpy as np
import pytest

from helpers import run_forward

pytestmark = pytest.mark.gpu


def _calls(n, w, inp):
    import torch
    from paper_2602_12675_amd import api
    for _ in range(n):
        run_forward(api, torch, inp, want_lse=False)
    torch.cuda.synchronize()


@pytest.fixture(scope="module")
def tiny():
    from paper_2602_12675_amd import workloads as W
    w = W.TINY
    return w, W.generate(w)


def test_every_call_is_bracketed(tiny):
    from paper_2602_12675_amd import api
    w, inp = tiny
    api.sla2_profile_begin(["block_sums", "topk", "kv_state", "kv_total", "attn"], 3)
    _calls(4, w, inp)                       # the fourth call is past max_calls
    got = api.sla2_profile_end()
    for name in ("block_sums", "topk", "kv_state", "kv_total", "attn"):
        ms, n = got[name]
        assert n == 3 and ms > 0.0, (name, got)
    assert "dense" not in got               # stages that never ran are not reported


def test_sampled_brackets_every_nth_call(tiny):
    from paper_2602_12675_amd import api
    w, inp = tiny
    api.sla2_profile_begin_sampled(["attn"], 10, 3)
    _calls(7, w, inp)                       # calls 1, 4, 7
    got = api.sla2_profile_end()
    assert got["attn"][1] == 3 and got["attn"][0] > 0.0
    api.sla2_profile_begin_sampled(["attn"], 2, 2)
    _calls(7, w, inp)                       # calls 1, 3 (5 and 7 are past max_calls)
    assert api.sla2_profile_end()["attn"][1] == 2


def test_bad_arguments(tiny):
    from paper_2602_12675_amd import api
    with pytest.raises(api.Sla2Error):
        api.sla2_profile_begin_sampled(["attn"], 4, 0)
    with pytest.raises(api.Sla2Error):
        api.sla2_profile_begin([], 4)
    api.sla2_profile_begin(["attn"], 1)
    with pytest.raises(api.Sla2Error):      # begin without end
        api.sla2_profile_begin(["attn"], 1)
    api.sla2_profile_end()


def test_backward_stages_are_bracketed():
    import torch
    from paper_2602_12675_amd import api, workloads as W
    from test_gpu_backward import run_fwd_bwd
    w = W.TINY.replace(name="prof-bwd", per_head_freq=True)
    inp = W.generate(w)
    alpha = np.full((w.H,), 0.5, dtype=np.float32)
    dout = np.ones((w.B, w.H, w.N, w.d), dtype=np.float32)
    api.sla2_profile_begin(["attn", "bwd_lists", "bwd_q", "bwd_kv", "bwd_rest"], 2)
    for _ in range(3):                      # a forward and a backward call each; the third pair is past max_calls
        run_fwd_bwd(api, torch, inp, alpha, False, True, dout)
    got = api.sla2_profile_end()
    # max_calls counts entry-point calls: the first forward and the first backward call are bracketed
    assert got["attn"][1] + got["bwd_q"][1] == 2, got
    assert got["bwd_q"][1] == got["bwd_kv"][1] == got["bwd_lists"][1]
    assert got["bwd_rest"][1] == 2 * got["bwd_q"][1]          # totals and finish
    assert all(ms > 0.0 for ms, n in got.values())
