"""fp64 CPU oracle for the fused dense-layer block.  TEST INFRASTRUCTURE ONLY.

    Y = LayerNorm(GELU_erf(X W^T + b)) * gamma + beta,   backward for dY.

This file is the parity reference that the GPU kernels are checked against.
It is deliberately slow and plain: every function is the mathematical
definition written out in numpy float64, one line per formula, with library
primitives (matmul, erfc, exp) as steps.  It shares no code with the GPU
path and must never be imported by it; only tests, the smoke check and the
benchmark's CPU-baseline leg may use it.

Conventions (paper, appendix "Robust Kernel Benchmark", linear backward task
definition): the linear step is `F.linear`, y = x W^T + b with W stored
[out_features, in_features]; the backward pass receives the upstream
gradient plus the saved tensors and returns the gradient of every input.
The paper defines a correct kernel as one that reproduces the torch
operator (appendix "Kernel Evaluation Environment"), so GELU is the exact
erf form and LayerNorm uses the biased variance with eps inside the root.

Pins (tests/test_oracle_pins.py): closed forms of Phi/phi/GELU against a
40-digit series evaluation, row invariants of the normalisation and of its
gradient, central finite differences of sum(dY*Y) for all five gradients,
the same composition through torch's float64 functional ops + autograd,
element-by-element Python loops on tiny shapes, and degenerate cases
(N = 1, W = 0, constant rows).  Nothing here is "parity unpinned".
"""
from __future__ import annotations

import math
from typing import Dict, Iterable, Optional

import numpy as np
from scipy.special import erfc

_SQRT2 = math.sqrt(2.0)
_INV_SQRT_2PI = 1.0 / math.sqrt(2.0 * math.pi)


def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float64)


# ---------------------------------------------------------------- GELU (erf)
def Phi(z):
    """Standard normal CDF.  erfc form: no cancellation for z << 0."""
    return 0.5 * erfc(-_f64(z) / _SQRT2)


def phi(z):
    """Standard normal density."""
    z = _f64(z)
    return np.exp(-0.5 * z * z) * _INV_SQRT_2PI


def gelu(z):
    """GELU(z) = z * Phi(z)  (exact form, not the tanh approximation)."""
    z = _f64(z)
    return z * Phi(z)


def gelu_grad(z):
    """d/dz [z Phi(z)] = Phi(z) + z phi(z)."""
    z = _f64(z)
    return Phi(z) + z * phi(z)


# ------------------------------------------------------------------- forward
def linear(X, W, b):
    """Z_ij = sum_k X_ik W_jk + b_j   (W is [N, K])."""
    return _f64(X) @ _f64(W).T + _f64(b)[None, :]


def row_stats(A, eps):
    """Per-row mean, biased variance (two-pass), and r = (var + eps)^-1/2."""
    A = _f64(A)
    mu = A.mean(axis=1)
    var = ((A - mu[:, None]) ** 2).mean(axis=1)
    rstd = 1.0 / np.sqrt(var + eps)
    return mu, var, rstd


def forward(X, W, b, gamma, beta, eps=1e-5) -> Dict[str, np.ndarray]:
    """Whole forward.  Returns Y and the tensors saved for backward."""
    Z = linear(X, W, b)
    A = gelu(Z)
    mu, _, rstd = row_stats(A, eps)
    Ahat = (A - mu[:, None]) * rstd[:, None]
    Y = Ahat * _f64(gamma)[None, :] + _f64(beta)[None, :]
    return {"Y": Y, "Z": Z, "mean": mu, "rstd": rstd}


# ------------------------------------------------------------------ backward
def backward_rows(dY, gamma, Z, mean, rstd) -> Dict[str, np.ndarray]:
    """Row-local part of the backward pass: everything up to dZ.

    g = dY*gamma;  c1 = mean_j g;  c2 = mean_j g*Ahat;
    dA = r (g - c1 - Ahat c2)     (from dAhat_j/dA_k = r[d_jk - 1/N - Ahat_j Ahat_k / N])
    dZ = dA * GELU'(Z)
    """
    dY, Z = _f64(dY), _f64(Z)
    mean, rstd = _f64(mean), _f64(rstd)
    A = gelu(Z)
    Ahat = (A - mean[:, None]) * rstd[:, None]
    g = dY * _f64(gamma)[None, :]
    c1 = g.mean(axis=1)
    c2 = (g * Ahat).mean(axis=1)
    dA = rstd[:, None] * (g - c1[:, None] - Ahat * c2[:, None])
    dZ = dA * gelu_grad(Z)
    return {"dZ": dZ, "Ahat": Ahat}


def backward(dY, X, W, gamma, Z, mean, rstd) -> Dict[str, np.ndarray]:
    """Whole backward given the saved tensors (Z, mean, rstd)."""
    dY = _f64(dY)
    rows = backward_rows(dY, gamma, Z, mean, rstd)
    dZ, Ahat = rows["dZ"], rows["Ahat"]
    return {
        "dX": dZ @ _f64(W),            # [M,N] x [N,K]
        "dW": dZ.T @ _f64(X),          # [N,M] x [M,K]
        "db": dZ.sum(axis=0),
        "dgamma": (dY * Ahat).sum(axis=0),
        "dbeta": dY.sum(axis=0),
        "dZ": dZ,
    }


def forward_backward(X, W, b, gamma, beta, dY, eps=1e-5) -> Dict[str, np.ndarray]:
    f = forward(X, W, b, gamma, beta, eps)
    g = backward(dY, X, W, gamma, f["Z"], f["mean"], f["rstd"])
    out = dict(f)
    out.update(g)
    return out


# ------------------------------------------------- large inputs, row by row
def forward_backward_streamed(X, W, b, gamma, beta, dY, eps=1e-5,
                              block_rows: int = 1024,
                              rows: Optional[Iterable[int]] = None,
                              keep_rows: Optional[Iterable[int]] = None
                              ) -> Dict[str, np.ndarray]:
    """Same result as `forward_backward`, bounded memory.

    Every step up to dZ is local to a row, and dW/db/dgamma/dbeta are sums
    over rows, so the rows are visited in blocks and the four sums are
    accumulated block by block; each block goes through `forward` and
    `backward` above unchanged.

    rows:      visit only these rows (sums then run over this subset only;
               exact whenever dY is zero on every other row).
    keep_rows: row indices whose Y, Z, dX rows are returned (default: none,
               only mean/rstd and the four sums are returned).
    """
    M = X.shape[0]
    N, K = W.shape
    row_idx = np.arange(M) if rows is None else np.asarray(sorted(set(int(r) for r in rows)))
    keep = set(int(r) for r in keep_rows) if keep_rows is not None else set()
    Wd, bd, gd, btd = _f64(W), _f64(b), _f64(gamma), _f64(beta)
    dW = np.zeros((N, K)); db = np.zeros(N); dgamma = np.zeros(N); dbeta = np.zeros(N)
    mean = np.full(M, np.nan); rstd = np.full(M, np.nan)
    kept = {"rows": [], "Y": [], "Z": [], "dX": []}
    for s in range(0, len(row_idx), block_rows):
        idx = row_idx[s:s + block_rows]
        Xb = _f64(np.asarray(X[idx]))
        dYb = _f64(np.asarray(dY[idx]))
        f = forward(Xb, Wd, bd, gd, btd, eps)
        g = backward(dYb, Xb, Wd, gd, f["Z"], f["mean"], f["rstd"])
        dW += g["dW"]; db += g["db"]; dgamma += g["dgamma"]; dbeta += g["dbeta"]
        mean[idx] = f["mean"]; rstd[idx] = f["rstd"]
        for local, r in enumerate(idx):
            if int(r) in keep:
                kept["rows"].append(int(r))
                kept["Y"].append(f["Y"][local]); kept["Z"].append(f["Z"][local])
                kept["dX"].append(g["dX"][local])
    out = {"dW": dW, "db": db, "dgamma": dgamma, "dbeta": dbeta, "mean": mean, "rstd": rstd}
    if keep:
        out["kept_rows"] = np.asarray(kept["rows"])
        for k in ("Y", "Z", "dX"):
            out["kept_" + k] = np.stack(kept[k])
    return out
