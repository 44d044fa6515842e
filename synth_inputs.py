"""Seeded synthetic inputs for the Skiparse-2D attention workloads.

Serves both the float64 oracle and the GPU library in tests and in the benchmark.  It holds no
arithmetic of the method itself: it only draws Q, K, V with the shapes and value distributions of
the workloads and rounds them to the storage type once.  Everything is generated on the CPU with
``torch.Generator(seed)`` so the two sides see identical bits.

The shapes stand in for the self-attention inputs of a Wan2.1-shaped video DiT (the paper's Sec. 4.1
model: 40 heads of 128 channels at 14B; 12 heads at the 1.3B size) on latent token grids of
81-frame 480x832 and 768x1280 video (T=21; H,W = pixels/16).  Real activations need the model's
weights, which are not available; i.i.d. N(0,1) values (optionally with a per-head gain on q and k
after a per-token normalisation, mimicking QK-norm layers) are used instead.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    heads: int
    D: int
    T: int
    H: int
    W: int
    s: int
    patterns: tuple
    dtype: str  # "f32" or "bf16": storage type of q, k, v
    seed: int
    qk_norm_gain: bool = False  # per-(token, head) normalisation of q,k + per-head gain 2^U(-1,1)

    @property
    def N(self) -> int:
        return self.T * self.H * self.W

    @property
    def Nsub(self) -> int:
        return self.N // (self.s * self.s)

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.D))

    def sparse_flops(self) -> float:
        """4 * units * Nsub^2 * D: QK^T and PV multiply-adds of one sparse call."""
        return 4.0 * self.B * self.heads * self.s * self.s * float(self.Nsub) ** 2 * self.D

    def dense_flops(self) -> float:
        return 4.0 * self.B * self.heads * float(self.N) ** 2 * self.D


WORKLOADS = {
    w.name: w
    for w in [
        Workload("tiny", 1, 2, 64, 2, 8, 8, 2, ("token", "group"), "f32", 0),
        Workload("480p", 1, 12, 128, 21, 30, 52, 2, ("token",), "bf16", 1, qk_norm_gain=True),
        Workload("768p", 1, 40, 128, 21, 48, 80, 2, ("token", "group"), "bf16", 2),
        Workload("hybrid", 1, 40, 128, 21, 48, 80, 2, ("token", "group"), "bf16", 3),
        Workload("fp8", 1, 40, 128, 21, 48, 80, 2, ("group",), "bf16", 4),
    ]
}


def make_shape(name, B, heads, D, T, H, W, s, dtype="bf16", seed=0, qk_norm_gain=False) -> Workload:
    """An ad-hoc workload (parity tests use small grids that still span several tiles)."""
    return Workload(name, B, heads, D, T, H, W, s, ("token", "group"), dtype, seed, qk_norm_gain)


def make_qkv(w: Workload):
    """Returns (q, k, v) CPU torch tensors of shape [B][N][heads][D] in the workload's storage dtype."""
    g = torch.Generator(device="cpu")
    g.manual_seed(w.seed)
    shape = (w.B, w.N, w.heads, w.D)
    out = []
    gains = None
    if w.qk_norm_gain:
        gains = torch.pow(2.0, torch.rand((2, w.heads), generator=g, dtype=torch.float32) * 2.0 - 1.0)
    for idx in range(3):
        x = torch.randn(shape, generator=g, dtype=torch.float32)
        if w.qk_norm_gain and idx < 2:
            x = x - x.mean(dim=-1, keepdim=True)
            x = x / x.std(dim=-1, keepdim=True, unbiased=False)
            x = x * gains[idx].view(1, 1, w.heads, 1)
        if w.dtype == "bf16":
            x = x.to(torch.bfloat16)
        out.append(x.contiguous())
    return tuple(out)


def make_dout(w: Workload) -> torch.Tensor:
    """Upstream gradient dL/dout for the backward pass: N(0,1) in the workload's storage dtype, seeded apart from q, k, v."""
    g = torch.Generator(device="cpu")
    g.manual_seed(w.seed + 1000)
    x = torch.randn((w.B, w.N, w.heads, w.D), generator=g, dtype=torch.float32)
    if w.dtype == "bf16":
        x = x.to(torch.bfloat16)
    return x.contiguous()


def as_oracle_array(x: torch.Tensor) -> np.ndarray:
    """View a CPU tensor as what the oracle takes: float32/float64 as is, bfloat16 as uint16 bit patterns."""
    if x.dtype == torch.bfloat16:
        return x.view(torch.int16).numpy().view(np.uint16)
    return x.numpy()


def sample_rows(w: Workload, per_unit: int, seed: int) -> np.ndarray:
    """(b, head, n) query positions: `per_unit` random tokens for every (batch, head), drawn uniformly
    over the whole grid (so that every subsequence of both patterns is hit), plus the first and last token."""
    rng = np.random.default_rng(seed)
    rows = []
    for b in range(w.B):
        for hd in range(w.heads):
            ns = rng.integers(0, w.N, size=per_unit)
            for n in list(ns) + [0, w.N - 1]:
                rows.append((b, hd, int(n)))
    return np.asarray(rows, dtype=np.int64)
