"""fp64 CPU oracle for the sibling operators that share the block's kernels.  TEST INFRASTRUCTURE ONLY.

Plain numpy float64 definitions, one line per formula, of the operators from the paper's task table (section on
the robust kernel benchmark, table of benchmark tasks) that the library builds on the same kernels as the fused
dense-layer block:

  * Linear + ReLU forward and backward (appendix "Highlighted CUDA Kernels: Code", "MNIST Linear-ReLU" forward
    kernel and "MNIST Linear-ReLU Backward Kernel": y = max(0, x W^T + b); the backward pass recomputes the
    pre-activation from x, W, b to build the activation mask, then forms the three linear-layer gradients from
    the masked upstream gradient);
  * LayerNorm forward (appendix "Highlighted CUDA Kernels: Analysis", Layernorm: per-row mean and variance, then
    normalise and apply the affine transform; torch semantics: biased variance, eps inside the root);
  * Llama RMSNorm forward ("Llama RMSNorm Forward Kernel" listing: y = x * rsqrt(mean(x^2) + eps) * w);
  * Llama feed-forward block forward (same appendix, LlamaFFW: three matrix products and a fused SiLU-multiply:
    y = (SiLU(x Wg^T) * (x Wu^T)) Wd^T, no biases).

Shares no code with the GPU path and must never be imported by it; only tests, the smoke check and the
benchmark's CPU-baseline leg may use it.  Pins: tests/test_siblings_oracle_pins.py (closed forms, invariants,
central finite differences, torch float64 functional ops and autograd, Python loops on tiny shapes, planted
mistakes).  Nothing here is "parity unpinned".
"""
from __future__ import annotations

from typing import Dict

import numpy as np


def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float64)


# ------------------------------------------------------------------ Linear + ReLU
def linear_relu_forward(X, W, b) -> Dict[str, np.ndarray]:
    """Z = X W^T + b (W is [N, K]);  Y = max(Z, 0)."""
    Z = _f64(X) @ _f64(W).T + _f64(b)[None, :]
    return {"Y": np.maximum(Z, 0.0), "Z": Z}


def linear_relu_backward(dY, X, W, b) -> Dict[str, np.ndarray]:
    """The pre-activation is recomputed from the inputs; the mask is Z > 0 (the derivative at 0 is taken as 0).
    G = dY * [Z > 0];  dX = G W;  dW = G^T X;  db = column sums of G."""
    X, W = _f64(X), _f64(W)
    Z = X @ W.T + _f64(b)[None, :]
    G = _f64(dY) * (Z > 0.0)
    return {"dX": G @ W, "dW": G.T @ X, "db": G.sum(axis=0), "G": G, "Z": Z}


# ------------------------------------------------------------------ LayerNorm forward
def layernorm_forward(A, gamma, beta, eps=1e-5) -> Dict[str, np.ndarray]:
    """Per row: mean, biased variance (two-pass), r = (var + eps)^-1/2;  Y = (A - mean) r gamma + beta."""
    A = _f64(A)
    mu = A.mean(axis=1)
    var = ((A - mu[:, None]) ** 2).mean(axis=1)
    rstd = 1.0 / np.sqrt(var + eps)
    Y = (A - mu[:, None]) * rstd[:, None] * _f64(gamma)[None, :] + _f64(beta)[None, :]
    return {"Y": Y, "mean": mu, "rstd": rstd}


# ------------------------------------------------------------------ RMSNorm forward
def rmsnorm_forward(A, weight, eps=1e-5) -> Dict[str, np.ndarray]:
    """Per row: ms = mean_j A_j^2;  Y = A (ms + eps)^-1/2 weight."""
    A = _f64(A)
    ms = (A * A).mean(axis=1)
    rrms = 1.0 / np.sqrt(ms + eps)
    return {"Y": A * rrms[:, None] * _f64(weight)[None, :], "rrms": rrms}


# ------------------------------------------------------------------ Llama feed-forward forward
def silu(z):
    """SiLU(z) = z * sigmoid(z) = z / (1 + exp(-z))."""
    z = _f64(z)
    return z / (1.0 + np.exp(-z))


def llama_ffn_forward(X, Wg, Wu, Wd) -> Dict[str, np.ndarray]:
    """G = X Wg^T, U = X Wu^T  ([M, H], Wg and Wu are [H, D]);  Hact = SiLU(G) * U;  Y = Hact Wd^T  (Wd is [D, H])."""
    X = _f64(X)
    G = X @ _f64(Wg).T
    U = X @ _f64(Wu).T
    Hact = silu(G) * U
    return {"Y": Hact @ _f64(Wd).T, "H": Hact, "G": G, "U": U}
