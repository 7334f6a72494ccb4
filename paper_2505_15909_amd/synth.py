"""Seeded synthetic inputs shaped like the paper's workloads.

The paper measures on the linear modules of Llama-3.1 8B / 70B / 405B (Section 3,
Section 4: four linear modules per Transformer layer; Section 5: generation
benchmarks).  Real weights are not available here, so tensors of the same shapes are
drawn from stated distributions.  This module holds *no* arithmetic of the method
(no scales, no rounding, no packing): it only produces fp16 tensors.  The GPU path
and the CPU checker both consume the very same tensors (one side gets a copy).
"""
from __future__ import annotations

import torch

# module name -> (K in, N out) ; module ids follow Section 4.2: 1=qkv 2=o 3=gate_up 4=down
LLAMA_8B = {"qkv": (4096, 6144), "o": (4096, 4096), "gate_up": (4096, 28672), "down": (14336, 4096)}
LLAMA_70B = {"qkv": (8192, 10240), "o": (8192, 8192), "gate_up": (8192, 57344), "down": (28672, 8192)}
LLAMA_405B = {"qkv": (16384, 18432), "o": (16384, 16384), "gate_up": (16384, 106496), "down": (53248, 16384)}
MODULE_ID = {"qkv": 1, "o": 2, "gate_up": 3, "down": 4}


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def normal_weight(N: int, K: int, std: float, seed: int, device="cpu") -> torch.Tensor:
    """fp16 [N, K] ~ N(0, std^2), drawn in fp32 then cast."""
    w = torch.randn(N, K, generator=_gen(device, seed), device=device, dtype=torch.float32)
    return (w * std).to(torch.float16)


def heavy_tail_weight(N: int, K: int, scale: float, seed: int, device="cpu",
                      df: int = 4, outlier_frac: float = 0.01, outlier_gain: float = 10.0) -> torch.Tensor:
    """fp16 [N, K]: scale * Student-t(df), then a fixed random subset of the *input
    columns* (outlier_frac of K) multiplied by outlier_gain -- the outlier-channel
    structure the paper's Section 2.2 motivates group-wise scaling with."""
    g = _gen(device, seed)
    z = torch.randn(N, K, generator=g, device=device, dtype=torch.float32)
    chi = torch.zeros(N, K, device=device, dtype=torch.float32)
    for _ in range(df):
        chi += torch.randn(N, K, generator=g, device=device, dtype=torch.float32) ** 2
    t = z / torch.sqrt(chi / df)
    n_out = max(1, int(round(outlier_frac * K)))
    cols = torch.randperm(K, generator=g, device=device)[:n_out]
    t[:, cols] *= outlier_gain
    return (t * scale).clamp_(-60000.0, 60000.0).to(torch.float16)


def activation(M: int, K: int, seed: int, device="cpu") -> torch.Tensor:
    """fp16 [M, K] ~ N(0, 1)."""
    a = torch.randn(M, K, generator=_gen(device, seed), device=device, dtype=torch.float32)
    return a.to(torch.float16)
