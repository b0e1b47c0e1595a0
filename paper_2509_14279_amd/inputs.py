"""Seeded synthetic inputs for the fused dense-layer block.

This module only draws random numbers and rounds them to the storage type.
It holds none of the operator's arithmetic, so both the GPU path's tests and
the CPU oracle's tests can be fed from it without sharing any of the method.

Conventions follow the paper's task definitions (appendix "Robust Kernel
Benchmark", linear task listing): the weight is stored [out_features,
in_features] as in `F.linear`, the bias is non-zero, and the backward pass
receives an upstream gradient of the output's shape.

Distribution reading: `N(a, s)` is taken as mean a, VARIANCE s, so
W ~ N(0, 1/K) has standard deviation K**-0.5, b ~ N(0, 0.02) has standard
deviation sqrt(0.02), gamma = 1 + N(0, 0.1), beta ~ N(0, 0.1), and
X ~ N(50, 100**2) has standard deviation 100.

Draw order with one CPU generator seeded by `seed`: X, W, b, gamma, beta, dY,
each as fp32 standard normals that are then scaled and shifted in fp32.  In
bf16 configurations every tensor (vectors included) is then rounded once to
the nearest bf16 value (ties to even) so that readers in either precision see
identical numbers.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict

import torch


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    dtype: str          # "f32" or "bf16": storage type of the matrices
    M: int
    K: int
    N: int
    seed: int
    x_mean: float = 0.0
    x_std: float = 1.0
    eps: float = 1e-5

    @property
    def gemm_flop(self) -> float:
        """Flop of the three contractions (forward, dX, dW): 6*M*N*K."""
        return 6.0 * self.M * self.N * self.K


# The five seeded configurations (seed = index).
CONFIGS = (
    Config("cfg0_f32_256x256x256", "f32", 256, 256, 256, seed=0),
    Config("cfg1_bf16_8192x1024x4096", "bf16", 8192, 1024, 4096, seed=1),
    Config("cfg2_f32_ragged_3001x771x1537", "f32", 3001, 771, 1537, seed=2),
    Config("cfg3_bf16_16384x4096x4096_shifted", "bf16", 16384, 4096, 4096, seed=3,
           x_mean=50.0, x_std=100.0),
    Config("cfg4_bf16_65536x2048x8192", "bf16", 65536, 2048, 8192, seed=4),
)


def custom(dtype: str, M: int, K: int, N: int, seed: int, **kw) -> Config:
    return Config(f"custom_{dtype}_{M}x{K}x{N}_s{seed}", dtype, M, K, N, seed, **kw)


def _round_to_storage(t: torch.Tensor, dtype: str) -> torch.Tensor:
    if dtype == "bf16":
        return t.to(torch.bfloat16).to(torch.float32)
    if dtype == "f32":
        return t
    raise ValueError(f"unknown dtype {dtype!r}")


def generate(cfg: Config, with_dY: bool = True) -> Dict[str, torch.Tensor]:
    """Return fp32 CPU tensors holding storage-representable values.

    Keys: X [M,K], W [N,K], b, gamma, beta [N], dY [M,N] (if requested).
    """
    g = torch.Generator(device="cpu")
    g.manual_seed(cfg.seed)
    M, K, N = cfg.M, cfg.K, cfg.N

    def randn(*shape):
        return torch.randn(*shape, generator=g, dtype=torch.float32)

    X = randn(M, K)
    if cfg.x_std != 1.0:
        X.mul_(cfg.x_std)
    if cfg.x_mean != 0.0:
        X.add_(cfg.x_mean)
    W = randn(N, K).mul_(1.0 / math.sqrt(K))
    b = randn(N).mul_(math.sqrt(0.02))
    gamma = randn(N).mul_(math.sqrt(0.1)).add_(1.0)
    beta = randn(N).mul_(math.sqrt(0.1))
    out = {"X": X, "W": W, "b": b, "gamma": gamma, "beta": beta}
    if with_dY:
        out["dY"] = randn(M, N)
    return {k: _round_to_storage(v, cfg.dtype) for k, v in out.items()}


def storage_torch_dtype(dtype: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


# ---------------------------------------------------------------- sibling operators (draws and rounding only)
def generate_norm(dtype: str, M: int, N: int, seed: int, mean: float = 0.5, std: float = 2.0) -> Dict[str, torch.Tensor]:
    """Inputs of the stand-alone row normalisations: A [M,N] ~ N(mean, std^2) rounded to the storage type; gamma
    (also the RMSNorm weight) = 1 + N(0, 0.1), beta ~ N(0, 0.1) in full fp32 (they are fp32 by contract).
    Draw order: A, gamma, beta."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    A = torch.randn(M, N, generator=g, dtype=torch.float32).mul_(std).add_(mean)
    gamma = torch.randn(N, generator=g, dtype=torch.float32).mul_(math.sqrt(0.1)).add_(1.0)
    beta = torch.randn(N, generator=g, dtype=torch.float32).mul_(math.sqrt(0.1))
    return {"A": _round_to_storage(A, dtype), "gamma": gamma, "beta": beta}


def generate_ffn(dtype: str, M: int, D: int, H: int, seed: int) -> Dict[str, torch.Tensor]:
    """Inputs of the gated feed-forward block: X [M,D] ~ N(0,1); Wg, Wu [H,D] ~ N(0, 1/D); Wd [D,H] ~ N(0, 1/H); all
    rounded to the storage type.  Draw order: X, Wg, Wu, Wd."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    X = torch.randn(M, D, generator=g, dtype=torch.float32)
    Wg = torch.randn(H, D, generator=g, dtype=torch.float32).mul_(1.0 / math.sqrt(D))
    Wu = torch.randn(H, D, generator=g, dtype=torch.float32).mul_(1.0 / math.sqrt(D))
    Wd = torch.randn(D, H, generator=g, dtype=torch.float32).mul_(1.0 / math.sqrt(H))
    return {k: _round_to_storage(v, dtype) for k, v in {"X": X, "Wg": Wg, "Wu": Wu, "Wd": Wd}.items()}
