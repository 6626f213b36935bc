"""ctypes binding of libsla2.so: same names as the C ABI in include/sla2.h.

Argument marshalling only - every step of the forward pass runs in the HIP
kernels.  torch is used for device memory (tensors own the buffers) and for the
current stream; nothing here computes.  If the library has not been built the
import of this module fails: there is no fallback.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsla2.so")

SLA2_F32, SLA2_BF16 = 0, 1
SLA2_QUANT_NONE, SLA2_QUANT_FP8, SLA2_QUANT_INT8, SLA2_QUANT_FP8_V = 0, 1, 2, 3
QUANT_MODES = {"none": SLA2_QUANT_NONE, "fp8": SLA2_QUANT_FP8, "int8": SLA2_QUANT_INT8,
               "fp8v": SLA2_QUANT_FP8_V}   # workload name -> sla2_quant
SLA2_FLAG_NO_SMOOTH_K = 1
SLA2_FLAG_SAVE_FOR_BACKWARD = 2
SLA2_OK, SLA2_EINVAL, SLA2_EUNSUPPORTED, SLA2_EWORKSPACE, SLA2_EALIAS, SLA2_EHIP = 0, -1, -2, -3, -4, -5

SLA2_STATIC_SCRATCH_BYTES = 32 << 20
EXPORTS = ("sla2_workspace_bytes", "sla2_workspace_layout", "sla2_num_selected", "sla2_router", "sla2_router_static",
           "sla2_router_soft", "sla2_forward", "sla2_backward", "sla2_dense_forward", "sla2_profile_begin", "sla2_profile_begin_sampled",
           "sla2_profile_end",
           "sla2_strerror", "sla2_version")

STAGES = ("block_sums", "topk", "kv_state", "kv_total", "attn", "dense",
          "bwd_lists", "bwd_q", "bwd_kv", "bwd_rest")   # sla2_stage


class Params(ctypes.Structure):
    """struct sla2_params"""
    _fields_ = [("B", ctypes.c_int), ("H", ctypes.c_int), ("N", ctypes.c_int), ("d", ctypes.c_int),
                ("block_q", ctypes.c_int), ("block_kv", ctypes.c_int), ("topk_frac", ctypes.c_float),
                ("dtype", ctypes.c_int), ("quant_mode", ctypes.c_int), ("router_w_per_head", ctypes.c_int),
                ("alpha_per_block", ctypes.c_int), ("flags", ctypes.c_uint),
                ("in_stride", ctypes.c_longlong * 3), ("out_stride", ctypes.c_longlong * 3)]


class WsLayout(ctypes.Structure):
    """struct sla2_ws_layout"""
    _fields_ = [(n, ctypes.c_size_t) for n in
                ("q_sum", "k_sum", "k_mean", "router_m", "block_idx", "h_total", "z_total",
                 "k_stats", "k_phi", "z_blocks", "k_fp8", "k_scale", "v_fp8", "v_scale", "partial",
                 "o_s", "o_l", "lse", "bwd", "total")]


if not os.path.exists(LIB_PATH):
    raise ImportError("libsla2.so is not built: run `python -m paper_2602_12675_amd.build` "
                      "(there is no CPU fallback)")
_lib = ctypes.CDLL(LIB_PATH)
_vp, _pp = ctypes.c_void_p, ctypes.POINTER(Params)
_lib.sla2_workspace_bytes.restype = ctypes.c_size_t
_lib.sla2_workspace_bytes.argtypes = [_pp]
_lib.sla2_workspace_layout.restype = ctypes.c_int
_lib.sla2_workspace_layout.argtypes = [_pp, ctypes.POINTER(WsLayout)]
_lib.sla2_num_selected.restype = ctypes.c_int
_lib.sla2_num_selected.argtypes = [_pp]
_lib.sla2_router.restype = ctypes.c_int
_lib.sla2_router.argtypes = [_pp, _vp, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.sla2_router_static.restype = ctypes.c_int
_lib.sla2_router_static.argtypes = [_pp, _vp, _vp, _vp, _vp, _vp]
_lib.sla2_router_soft.restype = ctypes.c_int
_lib.sla2_router_soft.argtypes = [_pp, _vp, _vp, _vp, ctypes.c_float, _vp, _vp, ctypes.c_size_t, _vp]
_lib.sla2_forward.restype = ctypes.c_int
_lib.sla2_forward.argtypes = [_pp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.sla2_backward.restype = ctypes.c_int
_lib.sla2_backward.argtypes = [_pp] + [_vp] * 10 + [ctypes.c_size_t, _vp]
_lib.sla2_dense_forward.restype = ctypes.c_int
_lib.sla2_dense_forward.argtypes = [_pp, _vp, _vp, _vp, _vp, _vp]
_lib.sla2_profile_begin.restype = ctypes.c_int
_lib.sla2_profile_begin.argtypes = [ctypes.c_uint, ctypes.c_int]
_lib.sla2_profile_begin_sampled.restype = ctypes.c_int
_lib.sla2_profile_begin_sampled.argtypes = [ctypes.c_uint, ctypes.c_int, ctypes.c_int]
_lib.sla2_profile_end.restype = ctypes.c_int
_lib.sla2_profile_end.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)]
_lib.sla2_strerror.restype = ctypes.c_char_p
_lib.sla2_strerror.argtypes = [ctypes.c_int]
_lib.sla2_version.restype = ctypes.c_int
_lib.sla2_version.argtypes = []


class Sla2Error(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__("libsla2: %s (%d)" % (sla2_strerror(status), status))


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else stream


def make_params(B, H, N, d, block_q, block_kv, topk_frac, dtype=SLA2_BF16, quant_mode=SLA2_QUANT_NONE,
                router_w_per_head=0, alpha_per_block=0, flags=0, in_stride=None, out_stride=None) -> Params:
    """in_stride / out_stride: (batch, head, token) element strides of q, k, v / of out; None = contiguous
    [B, H, N, d]."""
    p = Params(B, H, N, d, block_q, block_kv, topk_frac, dtype, quant_mode, router_w_per_head,
               alpha_per_block, flags)
    if in_stride is not None:
        p.in_stride[:] = [int(x) for x in in_stride]
    if out_stride is not None:
        p.out_stride[:] = [int(x) for x in out_stride]
    return p


def sla2_version() -> int:
    return _lib.sla2_version()


def sla2_strerror(status: int) -> str:
    return _lib.sla2_strerror(status).decode()


def sla2_workspace_bytes(params: Params) -> int:
    return _lib.sla2_workspace_bytes(ctypes.byref(params))


def sla2_workspace_layout(params: Params) -> WsLayout:
    out = WsLayout()
    rc = _lib.sla2_workspace_layout(ctypes.byref(params), ctypes.byref(out))
    if rc != SLA2_OK:
        raise Sla2Error(rc)
    return out


def sla2_num_selected(params: Params) -> int:
    rc = _lib.sla2_num_selected(ctypes.byref(params))
    if rc < 0:
        raise Sla2Error(rc)
    return rc


def sla2_router(params, q, k, router_w, block_idx, workspace, stream=None, check=True) -> int:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = _lib.sla2_router(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(router_w), _ptr(block_idx),
                          _ptr(workspace), ws_bytes, _stream(stream))
    if check and rc != SLA2_OK:
        raise Sla2Error(rc)
    return rc


def sla2_router_static(params, q, k, router_w, block_idx, stream=None, check=True) -> int:
    rc = _lib.sla2_router_static(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(router_w), _ptr(block_idx),
                                 _stream(stream))
    if check and rc != SLA2_OK:
        raise Sla2Error(rc)
    return rc


def sla2_router_soft(params, q, k, router_w, tau, mask_out, workspace, stream=None, check=True) -> int:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = _lib.sla2_router_soft(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(router_w), float(tau), _ptr(mask_out),
                               _ptr(workspace), ws_bytes, _stream(stream))
    if check and rc != SLA2_OK:
        raise Sla2Error(rc)
    return rc


def sla2_forward(params, q, k, v, router_w, alpha, out, block_idx=None, lse=None, workspace=None,
                 stream=None, check=True, ws_bytes=None) -> int:
    if ws_bytes is None:                               # a raw address needs its size spelled out
        ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = _lib.sla2_forward(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(v), _ptr(router_w), _ptr(alpha),
                           _ptr(out), _ptr(block_idx), _ptr(lse), _ptr(workspace), ws_bytes, _stream(stream))
    if check and rc != SLA2_OK:
        raise Sla2Error(rc)
    return rc


def sla2_backward(params, q, k, v, alpha, dout, dq, dk, dv, dalpha, workspace, stream=None, check=True,
                  ws_bytes=None) -> int:
    if ws_bytes is None:
        ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = _lib.sla2_backward(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(v), _ptr(alpha), _ptr(dout), _ptr(dq),
                            _ptr(dk), _ptr(dv), _ptr(dalpha), _ptr(workspace), ws_bytes, _stream(stream))
    if check and rc != SLA2_OK:
        raise Sla2Error(rc)
    return rc


def sla2_dense_forward(params, q, k, v, out, stream=None, check=True) -> int:
    rc = _lib.sla2_dense_forward(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _stream(stream))
    if check and rc != SLA2_OK:
        raise Sla2Error(rc)
    return rc


def sla2_profile_begin(stages, max_calls: int) -> None:
    """stages: iterable of names from STAGES."""
    mask = 0
    for name in stages:
        mask |= 1 << STAGES.index(name)
    rc = _lib.sla2_profile_begin(mask, max_calls)
    if rc != SLA2_OK:
        raise Sla2Error(rc)


def sla2_profile_begin_sampled(stages, max_calls: int, every: int) -> None:
    """As sla2_profile_begin, bracketing only every `every`-th call (max_calls of them)."""
    mask = 0
    for name in stages:
        mask |= 1 << STAGES.index(name)
    rc = _lib.sla2_profile_begin_sampled(mask, max_calls, every)
    if rc != SLA2_OK:
        raise Sla2Error(rc)


def sla2_profile_end() -> dict:
    """-> {stage name: (total ms, launches)} for the stages that ran."""
    ms = (ctypes.c_double * len(STAGES))()
    n = (ctypes.c_int * len(STAGES))()
    rc = _lib.sla2_profile_end(ms, n)
    if rc != SLA2_OK:
        raise Sla2Error(rc)
    return {STAGES[i]: (ms[i], n[i]) for i in range(len(STAGES)) if n[i]}


# ---- plumbing helpers for tests and the benchmark (no arithmetic) ------------------------------
def alloc_workspace(params: Params, device="cuda") -> torch.Tensor:
    n = sla2_workspace_bytes(params)
    if n == 0:
        raise Sla2Error(SLA2_EINVAL)
    return torch.empty(n, dtype=torch.uint8, device=device)


def workspace_view(workspace: torch.Tensor, offset: int, dtype: torch.dtype, shape) -> torch.Tensor:
    """A typed view of one region of the workspace (see sla2_ws_layout)."""
    count = 1
    for s in shape:
        count *= s
    nbytes = count * torch.empty((), dtype=dtype).element_size()
    return workspace[offset:offset + nbytes].view(dtype).view(*shape)


def to_device(arr, dtype_code: int, device="cuda") -> torch.Tensor:
    """numpy storage array (float32, or uint16 bf16 bit patterns) -> device tensor."""
    import numpy as np
    if dtype_code == SLA2_BF16:
        assert arr.dtype == np.uint16
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)
