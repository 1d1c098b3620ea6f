"""Seeded synthetic inputs shared by the GPU tests, the benchmark and the CPU oracle's tests.

This module holds no Lightning Attention arithmetic: it only draws random
tensors and evaluates the per-head decay schedules that are *input data* to
the attention path.  The paper's training corpus is private; these tensors
take only the shapes of its models (head dim 128; 8 / 16 / 32 heads for the
385M / 1B / 7B variants, App. A model table; pre-training length 8192, Sec. 4).

Distributions: Q, K, V i.i.d. N(0,1)/sqrt(D); dO i.i.d. N(0,1); drawn in fp32
on the CPU with one torch.Generator per tensor, then rounded to the run dtype.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch

BASE_SEED = 20230714


def decay_bench_rule(H: int) -> torch.Tensor:
    """lambda_h = exp(-2^(-8(h+1)/H)), h = 0..H-1, evaluated in fp64, rounded to fp32."""
    h = torch.arange(H, dtype=torch.float64)
    lam = torch.exp(-torch.pow(torch.tensor(2.0, dtype=torch.float64), -8.0 * (h + 1.0) / H))
    return lam.to(torch.float32)


def decay_paper_rule(H: int, layer: int = 0, n_layers: int = 1) -> torch.Tensor:
    """Eq. 2: lambda = exp(-(8h/H)(1 - l/L)) with h = 1..H; fp64 then fp32.

    The last layer (layer == n_layers) gives lambda = 1 for every head.
    """
    h = torch.arange(1, H + 1, dtype=torch.float64)
    lam = torch.exp(-(8.0 * h / H) * (1.0 - layer / n_layers))
    return lam.to(torch.float32)


def _randn(shape, seed: int, scale: float, dtype: torch.dtype) -> torch.Tensor:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    x = torch.randn(shape, generator=g, dtype=torch.float32)
    if scale != 1.0:
        x.mul_(scale)
    return x.to(dtype)


def make_qkv(Bt: int, H: int, N: int, D: int, dtype: torch.dtype, seed: int):
    """Q, K, V ~ N(0,1)/sqrt(D), shape [Bt,H,N,D], CPU tensors of `dtype`."""
    s = 1.0 / math.sqrt(D)
    shape = (Bt, H, N, D)
    return (_randn(shape, seed * 16 + 1, s, dtype),
            _randn(shape, seed * 16 + 2, s, dtype),
            _randn(shape, seed * 16 + 3, s, dtype))


def make_do(Bt: int, H: int, N: int, D: int, dtype: torch.dtype, seed: int) -> torch.Tensor:
    """dO ~ N(0,1), shape [Bt,H,N,D]."""
    return _randn((Bt, H, N, D), seed * 16 + 4, 1.0, dtype)


def make_gate(Bt: int, H: int, N: int, D: int, dtype: torch.dtype, seed: int) -> torch.Tensor:
    """Gate U ~ N(0,1), shape [Bt,H,N,D] (a projection of normalised activations)."""
    return _randn((Bt, H, N, D), seed * 16 + 9, 1.0, dtype)


def make_qkv_dkdv(Bt: int, H: int, N: int, Dk: int, Dv: int, dtype: torch.dtype, seed: int):
    """Q, K ~ N(0,1)/sqrt(Dk) of shape [Bt,H,N,Dk] and V ~ N(0,1)/sqrt(Dv) of shape [Bt,H,N,Dv]."""
    sk, sv = 1.0 / math.sqrt(Dk), 1.0 / math.sqrt(Dv)
    return (_randn((Bt, H, N, Dk), seed * 16 + 1, sk, dtype),
            _randn((Bt, H, N, Dk), seed * 16 + 2, sk, dtype),
            _randn((Bt, H, N, Dv), seed * 16 + 3, sv, dtype))


def make_preact(Bt: int, H: int, N: int, D: int, dtype: torch.dtype, seed: int, which: int = 0) -> torch.Tensor:
    """Pre-activation query (which = 0) or key (which = 1) projections X W ~ N(0,1), shape
    [Bt,H,N,D]: what the swish of Eq. 2 is applied to (normalised activations times a
    variance-preserving projection)."""
    return _randn((Bt, H, N, D), seed * 16 + 10 + which, 1.0, dtype)


def make_theta(H: int, D: int, seed: int) -> torch.Tensor:
    """LRPE-d angles, fp32 [H,D].  The paper only says they are learnable; these follow the
    usual geometric ladder of rotary encodings, theta_d = 10000^(-d/D), the same for every
    head up to a seeded +-10 % jitter standing in for what training would have moved."""
    d = torch.arange(D, dtype=torch.float64)
    base = torch.pow(torch.tensor(10000.0, dtype=torch.float64), -d / D)
    g = torch.Generator(device="cpu")
    g.manual_seed(seed * 16 + 12)
    jitter = 1.0 + 0.1 * (2.0 * torch.rand((H, D), generator=g, dtype=torch.float64) - 1.0)
    return (base[None, :] * jitter).to(torch.float32)


def make_step_qkv(Bt: int, H: int, D: int, dtype: torch.dtype, seed: int, step: int):
    """One decode token per (b,h): q, k, v ~ N(0,1)/sqrt(D), shape [Bt,H,D]."""
    s = 1.0 / math.sqrt(D)
    base = seed * 16 + 5
    return (_randn((Bt, H, D), base + 3 * 65536 * step + 0, s, dtype),
            _randn((Bt, H, D), base + 3 * 65536 * step + 65536, s, dtype),
            _randn((Bt, H, D), base + 3 * 65536 * step + 2 * 65536, s, dtype))


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: torch.dtype
    Bt: int
    H: int
    N: int
    D: int
    block: int          # 0 = library's choice
    backward: bool
    seed: int


# The measured configurations (index = position in the benchmark's config list).
CONFIGS = {
    "cfg1_fp32_small": Workload("cfg1_fp32_small", torch.float32, 1, 2, 256, 64, 64, False, BASE_SEED + 0),
    "cfg2_385m": Workload("cfg2_385m", torch.bfloat16, 8, 8, 2048, 128, 0, True, BASE_SEED + 1),
    "cfg2_385m_fp32": Workload("cfg2_385m_fp32", torch.float32, 8, 8, 2048, 128, 0, True, BASE_SEED + 1),
    "cfg_1b": Workload("cfg_1b", torch.bfloat16, 8, 16, 2048, 128, 0, True, BASE_SEED + 5),
    "cfg3_7b": Workload("cfg3_7b", torch.bfloat16, 4, 32, 8192, 128, 0, True, BASE_SEED + 2),
}
LONG_CONTEXT_N = (4096, 8192, 16384, 32768, 65536)   # Bt=1, H=32, D=128, bf16
LONG_CONTEXT_SEED = BASE_SEED + 3
DECODE = dict(Bt=64, H=32, D=128, prefix=1024, steps=512, seed=BASE_SEED + 4)
