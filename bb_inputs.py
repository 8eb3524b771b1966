"""Seeded synthetic inputs for the five benchmark configurations.

This module serves both the CPU oracle and the GPU path and therefore holds
none of the method's arithmetic: it only draws random tensors and rounds them
to bf16.  All tensors are CPU torch bf16 tensors; ``bits()`` gives the uint16
view the oracle consumes.

Recipe (one ``torch.Generator`` per configuration, seed 0 unless overridden;
tensors are drawn in fp32 in the fixed order X, g, W1, W3, W2 -- resp.
X, gamma, beta, W -- and rounded to nearest-even bf16; "N(a, b)" means mean a,
VARIANCE b):

  c1  FFN  M=64   D=256  F=704    X~N(0,1)            eps=1e-6
  c2  FFN  M=16   D=4096 F=11008  X~Student-t(nu=4)   eps=1e-6   (decode)
  c3  FFN  M=2048 D=4096 F=11008  X~N(0,1)            eps=1e-5   (prefill)
  c4  FFN  M=4096 D=8192 F=28672  X~N(0,1), round(0.01*D) columns x20, eps=1e-5
  c5  LN   M=8192 D=4096 N=16384  X~N(2,3), gamma~U(.5,1.5), beta~N(0,.1), eps=1e-5

  g, gamma ~ U(0.5, 1.5);  W1, W3, W ~ N(0, 1/D);  W2 ~ N(0, 1/F).
Student-t(4) is z / sqrt(chi2_4 / 4) with chi2_4 the sum of four squared
normals from the same generator.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, Optional

import torch


@dataclass(frozen=True)
class Config:
    name: str
    op: str            # "ffn" or "ln"
    M: int
    D: int
    F: int             # hidden size (ffn) or output size N (ln)
    eps: float
    x_dist: str        # "normal", "student4", "outlier_cols", "normal_2_3"
    note: str


CONFIGS: Dict[str, Config] = {
    "c1": Config("c1", "ffn", 64, 256, 704, 1e-6, "normal", "smoke / parity"),
    "c2": Config("c2", "ffn", 16, 4096, 11008, 1e-6, "student4", "decode, HBM bound"),
    "c3": Config("c3", "ffn", 2048, 4096, 11008, 1e-5, "normal", "prefill, MFMA bound"),
    "c4": Config("c4", "ffn", 4096, 8192, 28672, 1e-5, "outlier_cols", "large block"),
    "c5": Config("c5", "ln", 8192, 4096, 16384, 1e-5, "normal_2_3", "LayerNorm->matmul"),
}


def _randn(gen, *shape):
    return torch.randn(*shape, generator=gen, dtype=torch.float32)


def _draw_x(gen, M, D, dist):
    if dist == "normal":
        return _randn(gen, M, D)
    if dist == "student4":
        z = _randn(gen, M, D)
        chi2 = (_randn(gen, 4, M, D) ** 2).sum(dim=0)
        return z / torch.sqrt(chi2 / 4.0)
    if dist == "outlier_cols":
        x = _randn(gen, M, D)
        ncol = int(round(0.01 * D))
        cols = torch.randperm(D, generator=gen)[:ncol]
        x[:, cols] *= 20.0
        return x
    if dist == "normal_2_3":
        return 2.0 + math.sqrt(3.0) * _randn(gen, M, D)
    raise ValueError(dist)


def _uniform(gen, n, lo, hi):
    return lo + (hi - lo) * torch.rand(n, generator=gen, dtype=torch.float32)


def make_ffn(M: int, D: int, F: int, seed: int = 0, x_dist: str = "normal"):
    """X [M,D], g [D], W1 [D,F], W3 [D,F], W2 [F,D] as CPU bf16 tensors."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    X = _draw_x(gen, M, D, x_dist)
    g = _uniform(gen, D, 0.5, 1.5)
    W1 = _randn(gen, D, F) / math.sqrt(D)
    W3 = _randn(gen, D, F) / math.sqrt(D)
    W2 = _randn(gen, F, D) / math.sqrt(F)
    return tuple(t.to(torch.bfloat16).contiguous() for t in (X, g, W1, W3, W2))


def make_ln(M: int, D: int, N: int, seed: int = 0, x_dist: str = "normal_2_3"):
    """X [M,D], gamma [D], beta [D], W [D,N] as CPU bf16 tensors."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    X = _draw_x(gen, M, D, x_dist)
    gamma = _uniform(gen, D, 0.5, 1.5)
    beta = math.sqrt(0.1) * _randn(gen, D)
    W = _randn(gen, D, N) / math.sqrt(D)
    return tuple(t.to(torch.bfloat16).contiguous() for t in (X, gamma, beta, W))


def make_attn(B: int, M: int, N: int, d: int, dv: int, seed: int = 0, q_scale: float = 1.0):
    """Q [B,M,d], K [B,N,d], V [B,N,dv] as CPU bf16 tensors, all N(0,1) (Q times
    q_scale): scores Q K^T / sqrt(d) then have unit variance, like attention
    logits of a trained model at initialisation."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    Q = q_scale * torch.randn(B, M, d, generator=gen, dtype=torch.float32)
    K = torch.randn(B, N, d, generator=gen, dtype=torch.float32)
    V = torch.randn(B, N, dv, generator=gen, dtype=torch.float32)
    return tuple(t.to(torch.bfloat16).contiguous() for t in (Q, K, V))


def make_config(name: str, seed: int = 0, M: Optional[int] = None):
    """Inputs of a named configuration (optionally with fewer/more rows)."""
    c = CONFIGS[name]
    m = c.M if M is None else M
    if c.op == "ffn":
        return make_ffn(m, c.D, c.F, seed, c.x_dist)
    return make_ln(m, c.D, c.F, seed, c.x_dist)


def bits(t: torch.Tensor):
    """uint16 numpy view (bf16 bit patterns) of a CPU bf16 tensor."""
    return t.contiguous().view(torch.uint16).numpy()
