"""Host-only checks that the tolerance forms used by the GPU parity tests have teeth and are attainable.

For LayerNorm rows of one or two elements the backward outputs dX, dW, db are cancellation residues (of order
eps/var of their terms), so with bf16 storage they are held to `bar + c u_bf16 S` with S the magnitude of the
cancelling terms (harness.check_bf16_cancelling).  Here, entirely on the CPU: an implementation that follows the
definition but keeps the pre-activation in bf16 (emulated with the oracle on a rounded Z) stays inside that bound,
and a copy of the oracle's row step with a planted mistake (a dropped term, a wrong sign) falls outside it."""
import numpy as np
import pytest
import torch

from oracle import fdl_oracle as O
from paper_2509_14279_amd import inputs as I
import harness as H


def bf16_round(a: np.ndarray) -> np.ndarray:
    return torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16).float().numpy().astype(np.float64)


def backward_with(n, Z, mean, rstd, row_step):
    rows = row_step(n["dY"], n["gamma"], Z, mean, rstd)
    dZ = rows["dZ"]
    return {"dX": dZ @ n["W"], "dW": dZ.T @ n["X"], "db": dZ.sum(axis=0)}


def rows_drop_c2(dY, gamma, Z, mean, rstd):
    A = O.gelu(Z); Ahat = (A - mean[:, None]) * rstd[:, None]
    g = dY * gamma[None, :]; c1 = g.mean(axis=1)
    return {"dZ": rstd[:, None] * (g - c1[:, None]) * O.gelu_grad(Z)}                      # planted: no Ahat c2 term


def rows_wrong_sign(dY, gamma, Z, mean, rstd):
    A = O.gelu(Z); Ahat = (A - mean[:, None]) * rstd[:, None]
    g = dY * gamma[None, :]; c1 = g.mean(axis=1); c2 = (g * Ahat).mean(axis=1)
    return {"dZ": rstd[:, None] * (g - c1[:, None] + Ahat * c2[:, None]) * O.gelu_grad(Z)}   # planted: + instead of -


@pytest.mark.parametrize("shape", [(2, 2, 2), (17, 5, 2), (33, 1, 1), (9, 4, 1)])
def test_condition_aware_bound_accepts_bf16_storage_and_rejects_planted_mistakes(shape):
    M, K, N = shape
    cfg = I.custom("bf16", M, K, N, seed=300 + M + K + N)
    n = {k: v.numpy().astype(np.float64) for k, v in I.generate(cfg).items()}
    ref = O.forward_backward(n["X"], n["W"], n["b"], n["gamma"], n["beta"], n["dY"], cfg.eps)
    S = H.backward_term_scale(n, ref, cfg.eps)
    # an honest bf16 implementation: pre-activation stored rounded, statistics of the stored value, outputs rounded
    Zr = bf16_round(ref["Z"])
    mu, _, rs = O.row_stats(O.gelu(Zr), cfg.eps)
    mu32, rs32 = mu.astype(np.float32).astype(np.float64), rs.astype(np.float32).astype(np.float64)
    honest = backward_with(n, Zr, mu32, rs32, lambda *a: O.backward_rows(*a))
    for k in ("dX", "dW", "db"):
        got = bf16_round(honest[k]) if k != "db" else honest[k].astype(np.float32).astype(np.float64)
        H.check_bf16_cancelling(k, got, ref[k], S[k])
    if N == 1:
        return      # with one element per row g - c1 is identically zero and Ahat is zero: every variant gives dZ = 0
    for row_step in (rows_drop_c2, rows_wrong_sign):
        wrong = backward_with(n, Zr, mu32, rs32, row_step)
        with pytest.raises(AssertionError):
            for k in ("dX", "dW", "db"):
                H.check_bf16_cancelling(k, wrong[k], ref[k], S[k])


def test_ratio_log_records_every_bf16_comparison():
    H.RATIO_LOG.clear()
    H.set_ratio_label("case")
    r = H.check_bf16("t", np.array([1.0, 2.01]), np.array([1.0, 2.0]))
    assert H.RATIO_LOG == [("case", "t", r)] and abs(r - 0.005) < 1e-12
    with pytest.raises(AssertionError):
        H.check_bf16("t", np.array([1.0, 2.1]), np.array([1.0, 2.0]))
