"""Seeded synthetic video-DiT-shaped attention inputs.

This module holds none of the method's arithmetic: it only draws Q, K, V.  It
is the one module that the CPU oracle's tests and the HIP path's tests both
use, so that the two sides read identical bf16 bytes.

Recipe (stands in for the self-attention inputs of a video diffusion
transformer; the paper measures on real model activations, which are not
available here):
  * tokens lie on a (frames x height x width) latent grid in raster order;
    position p = (f/(F-1), y/(Hg-1), x/(Wg-1)) in [0,1]^3 (a size-1 axis maps
    to 0), multiplied by 3.0;
  * per head h a frequency matrix W_h in R^{64x3} ~ N(0,1), shared by Q and K;
    phi(p) = [cos(W_h p), sin(W_h p)] in R^128, so q.k/sqrt(d) peaks at
    64/sqrt(128) ~ 5.66 for coincident positions and decays with distance
    (diagonal / multi-diagonal tile structure);
  * Q0 = phi + 0.3 N(0,1), K0 = phi + 0.3 N(0,1) (independent), V0 ~ N(0,1);
  * optional text tokens appended after the video tokens: Q, K, V i.i.d. N(0,1);
  * per denoising step every tensor drifts as
    X_t = sqrt(0.98) X_{t-1} + sqrt(0.02) N(0,1) on an fp32 master copy; the
    bf16 rounding of X_t is what is handed out.
"""
from __future__ import annotations

import dataclasses
import math

import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    heads: int
    grid: tuple          # (frames, height, width) of the latent grid
    text_tokens: int = 0
    steps: int = 1
    head_dim: int = 128
    seed: int = 20251111

    @property
    def video_tokens(self) -> int:
        return self.grid[0] * self.grid[1] * self.grid[2]

    @property
    def seqlen(self) -> int:
        return self.video_tokens + self.text_tokens

    @property
    def protect(self) -> tuple:
        """(start, length) of the token range that must never be skipped."""
        return (self.video_tokens, self.text_tokens) if self.text_tokens else (0, 0)

    def dense_flops(self) -> float:
        """4 * B * H * N^2 * d: the dense-equivalent work of one attention call."""
        return 4.0 * self.batch * self.heads * float(self.seqlen) ** 2 * self.head_dim


# The five workloads of the benchmark definition.
WORKLOADS = {
    "tiny": Workload("tiny", 1, 2, (2, 32, 32), steps=4, seed=20251112),
    "wan1.3b_dense": Workload("wan1.3b_dense", 1, 12, (21, 30, 52), steps=1, seed=20251113),
    "wan1.3b_sweep": Workload("wan1.3b_sweep", 1, 12, (21, 30, 52), steps=10, seed=20251114),
    "wan14b": Workload("wan14b", 1, 40, (21, 60, 60), steps=50, seed=20251115),
    "longvideo": Workload("longvideo", 1, 24, (33, 45, 80), text_tokens=256, steps=30, seed=20251116),
}


def _positions(grid, device):
    F, Hg, Wg = grid
    def axis(n):
        if n == 1:
            return torch.zeros(1, device=device)
        return torch.arange(n, device=device, dtype=torch.float32) / float(n - 1)
    f, y, x = torch.meshgrid(axis(F), axis(Hg), axis(Wg), indexing="ij")
    return torch.stack([f.reshape(-1), y.reshape(-1), x.reshape(-1)], dim=1) * 3.0  # [Nv,3]


class DriftSequence:
    """Iterator over the denoising steps of one workload: each ``next()`` yields (q, k, v) as bf16
    tensors of shape [B,H,N,d] (contiguous) on ``device``."""

    def __init__(self, wl: Workload, device="cpu"):
        self.wl = wl
        self.device = torch.device(device)
        self.gen = torch.Generator(device=self.device)
        self.gen.manual_seed(wl.seed)
        self.t = -1
        self.master = None

    def _randn(self, *shape):
        return torch.randn(*shape, generator=self.gen, device=self.device, dtype=torch.float32)

    def _initial(self):
        wl = self.wl
        B, H, d = wl.batch, wl.heads, wl.head_dim
        Nv, N = wl.video_tokens, wl.seqlen
        nf = d // 2
        pos = _positions(wl.grid, self.device)                      # [Nv,3]
        W = self._randn(H, nf, 3)                                   # per-head frequencies
        ang = torch.einsum("hfk,nk->hnf", W, pos)                   # [H,Nv,nf]
        phi = torch.cat([torch.cos(ang), torch.sin(ang)], dim=2)    # [H,Nv,d]
        del ang
        out = []
        for name in ("q", "k", "v"):
            x = torch.empty(B, H, N, d, device=self.device, dtype=torch.float32)
            if name == "v":
                x[:, :, :Nv] = self._randn(B, H, Nv, d)
            else:
                x[:, :, :Nv] = phi.unsqueeze(0) + 0.3 * self._randn(B, H, Nv, d)
            if wl.text_tokens:
                x[:, :, Nv:] = self._randn(B, H, wl.text_tokens, d)
            out.append(x)
        return out

    def __iter__(self):
        return self

    def __next__(self):
        self.t += 1
        if self.master is None:
            self.master = self._initial()
        else:
            a, b = math.sqrt(0.98), math.sqrt(0.02)
            for x in self.master:
                x.mul_(a).add_(self._randn(*x.shape), alpha=b)
        return tuple(x.to(torch.bfloat16) for x in self.master)


def bf16_bits(t: torch.Tensor):
    """bf16 tensor (any device) -> uint16 numpy array of its bit patterns on the host."""
    import numpy as np
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
