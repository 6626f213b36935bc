"""Seeded synthetic workloads shaped like the paper's video-diffusion attention.

This module only draws random numbers and lays tensors out; it holds none of
the method's arithmetic and is the one piece shared by the HIP path's tests,
the benchmark and the CPU oracle's tests.  numpy only - it imports neither the
HIP binding nor the oracle.

The paper's own tensors are Q, K, V captured from Wan2.1 attention layers
(Sec. 9.1 of the paper, "Setup"), which are not available.  The stand-ins keep
what the method relies on: the shapes of the two models (N = 32,760 tokens on a
21 x 30 x 52 latent grid with 12 heads, N = 75,600 on 21 x 45 x 80 with 40
heads, d = 128) and the similarity of neighbouring tokens that makes pooled
scores informative (Sec. 4): every channel is unit Gaussian noise plus a
0.5-scaled sinusoid of the token's (t, y, x) grid position.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    grid: tuple            # (T, Y, X) latent grid; N = T*Y*X + extra_tokens
    d: int
    block_q: int
    block_kv: int
    topk_frac: float
    dtype: str             # storage type of q, k, v, out: "f32" | "bf16"
    quant: str             # "none" | "fp8" | "int8" | "fp8v" (FP8 with V quantised too)
    seed: int
    per_head_freq: bool    # False: f = (1,1,1); True: f ~ U[0.5, 4) per head and axis
    extra_tokens: int = 0  # tokens appended after the grid (ragged-tail cases)

    @property
    def N(self) -> int:
        return self.grid[0] * self.grid[1] * self.grid[2] + self.extra_tokens

    @property
    def T_m(self) -> int:
        return -(-self.N // self.block_q)

    @property
    def T_n(self) -> int:
        return -(-self.N // self.block_kv)

    @property
    def k(self) -> int:
        return max(0, min(self.T_n, int(math.floor(self.topk_frac * self.T_n + 0.5))))

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five configurations the benchmark definition names.
TINY = Workload("tiny", 1, 2, (4, 16, 16), 64, 64, 64, 0.125, "f32", "none", 0, False)
WAN_1P3B_95 = Workload("wan1.3b-95", 1, 12, (21, 30, 52), 128, 128, 64, 0.05, "bf16", "none", 0, True)
WAN_1P3B_97_FP8 = Workload("wan1.3b-97-fp8", 1, 12, (21, 30, 52), 128, 128, 64, 0.03, "bf16", "fp8", 0, True)
WAN_14B_97_FP8 = Workload("wan14b-97-fp8", 1, 40, (21, 45, 80), 128, 128, 64, 0.03, "bf16", "fp8", 1, True)
SWEEP_BASE = Workload("wan14b-sweep", 2, 40, (21, 45, 80), 128, 128, 64, 0.03, "bf16", "none", 1, True)
SWEEP_TOPK = (0.15, 0.10, 0.05, 0.03, 0.01)

# Beyond the five: image-generation-sized inputs (Sec. 1 names image models next to video ones): a 64 x 64
# latent grid, 4,096 tokens, 90 % sparsity, FP8 sparse branch; d = 128 with 128-row query blocks and d = 64
# with 64-row query blocks.
IMAGE_DIT_4K = Workload("image-dit-4k", 2, 24, (1, 64, 64), 128, 128, 64, 0.10, "bf16", "fp8", 2, True)
IMAGE_DIT_4K_D64 = Workload("image-dit-4k-d64", 2, 16, (1, 64, 64), 64, 64, 64, 0.10, "bf16", "fp8", 2, True)

CONFIGS = {w.name: w for w in (TINY, WAN_1P3B_95, WAN_1P3B_97_FP8, WAN_14B_97_FP8, SWEEP_BASE,
                               IMAGE_DIT_4K, IMAGE_DIT_4K_D64)}


@dataclasses.dataclass
class Inputs:
    workload: Workload
    q: np.ndarray          # [B,H,N,d] float32, or uint16 holding bf16 bit patterns
    k: np.ndarray
    v: np.ndarray
    router_w: np.ndarray   # [2,d,d] float32: Wq, Wk, each [d_in, d_out]
    alpha: np.ndarray      # [H] float32

    def values(self, name: str, b: int, h: int) -> np.ndarray:
        """One head of q / k / v as float64 holding exactly the stored values."""
        return stored_values(getattr(self, name)[b, h]).astype(np.float64)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even.  Inputs
    are finite."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(u: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def stored_values(a: np.ndarray) -> np.ndarray:
    """float32 view of the values an array of stored elements holds."""
    return bf16_bits_to_f32(a) if a.dtype == np.uint16 else np.asarray(a, dtype=np.float32)


def grid_positions(w: Workload) -> np.ndarray:
    """[N,3] normalised (t/T, y/Y, x/X) of token n = (t*Y + y)*X + x; appended
    tokens continue at t = T, T+1, ... with y = x = 0."""
    T, Y, X = w.grid
    n = np.arange(T * Y * X)
    pos = np.stack([(n // (Y * X)) / T, ((n // X) % Y) / Y, (n % X) / X], axis=1)
    if w.extra_tokens:
        ext = np.stack([(T + np.arange(w.extra_tokens)) / T,
                        np.zeros(w.extra_tokens), np.zeros(w.extra_tokens)], axis=1)
        pos = np.concatenate([pos, ext], axis=0)
    return pos


def generate(w: Workload) -> Inputs:
    """Draw one input set.  Fixed draw order from numpy.random.default_rng(seed):
    Q noise, K noise, V noise, frequencies, phases, Wq, Wk, alpha.

      X_s[b,h,n,c] = g + 0.5 sin(2 pi (f_t t/T + f_y y/Y + f_x x/X) + psi_{s,h,c}),
      g ~ N(0,1) iid, psi ~ U[0, 2 pi) per (tensor, head, channel),
      Wq, Wk ~ N(0, 1/d) (float32, shared by heads), alpha_h ~ U(0,1).
    """
    rng = np.random.default_rng(w.seed)
    B, H, N, d = w.B, w.H, w.N, w.d
    noise = [rng.standard_normal((B, H, N, d), dtype=np.float32) for _ in range(3)]
    if w.per_head_freq:
        freq = rng.uniform(0.5, 4.0, size=(H, 3))
    else:
        freq = np.ones((H, 3))
    psi = rng.uniform(0.0, 2.0 * math.pi, size=(3, H, d))
    Wq = (rng.standard_normal((d, d)) / math.sqrt(d)).astype(np.float32)
    Wk = (rng.standard_normal((d, d)) / math.sqrt(d)).astype(np.float32)
    alpha = rng.uniform(0.0, 1.0, size=(H,)).astype(np.float32)

    pos = grid_positions(w)                                   # [N,3]
    arg = 2.0 * math.pi * (pos @ freq.T)                      # [N,H]
    sin_a = np.sin(arg).T[:, :, None].astype(np.float32)      # [H,N,1]
    cos_a = np.cos(arg).T[:, :, None].astype(np.float32)
    out = []
    for s in range(3):
        # sin(a + psi) = sin a cos psi + cos a sin psi
        cp = np.cos(psi[s])[:, None, :].astype(np.float32)    # [H,1,d]
        sp = np.sin(psi[s])[:, None, :].astype(np.float32)
        x = noise[s]
        for b in range(B):
            x[b] += np.float32(0.5) * (sin_a * cp + cos_a * sp)
        out.append(f32_to_bf16_bits(x) if w.dtype == "bf16" else x)
        noise[s] = None
    return Inputs(w, out[0], out[1], out[2], np.stack([Wq, Wk]), alpha)
