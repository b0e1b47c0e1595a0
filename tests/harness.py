"""Shared helpers for the GPU parity tests: run the HIP path through the C ABI on
seeded inputs and compare with the fp64 oracle under the stated tolerances."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from paper_2509_14279_amd import inputs as I

GUARD = 4096  # bytes of sentinel on each side of every output buffer
SENTINEL = 0x5A


class Guarded:
    """A device buffer with sentinel bytes before and after the payload."""

    def __init__(self, shape, dtype, device="cuda"):
        self.shape = tuple(shape)
        self.dtype = dtype
        n = int(np.prod(self.shape)) if len(self.shape) else 1
        self.nbytes = n * torch.empty((), dtype=dtype).element_size()
        pad = (-self.nbytes) % 16
        self.raw = torch.full((GUARD + self.nbytes + pad + GUARD,), SENTINEL, dtype=torch.uint8, device=device)
        self.view = self.raw[GUARD:GUARD + self.nbytes].view(dtype).view(self.shape)
        assert self.view.data_ptr() % 16 == 0

    def intact(self) -> bool:
        head = self.raw[:GUARD]
        tail = self.raw[GUARD + self.nbytes:]
        return bool((head == SENTINEL).all().item() and (tail == SENTINEL).all().item())


def run_fdl(cfg: I.Config, t: Dict[str, torch.Tensor], backward: bool = True, check_guards: bool = True,
            stream: Optional[torch.cuda.Stream] = None) -> Dict[str, torch.Tensor]:
    """Forward (+ backward) through libfdl on cuda:0.  `t` holds fp32 CPU tensors of storage-exact values.
    Returns device tensors (storage dtype for matrices, fp32 for vectors)."""
    from paper_2509_14279_amd import api

    dt = I.storage_torch_dtype(cfg.dtype)
    dev = "cuda"
    M, K, N = cfg.M, cfg.K, cfg.N
    X = t["X"].to(dev, dt); W = t["W"].to(dev, dt)
    b = t["b"].to(dev); gamma = t["gamma"].to(dev); beta = t["beta"].to(dev)
    ws_bytes = api.fdl_workspace_bytes(cfg.dtype, M, K, N)
    assert ws_bytes > 0
    ws = Guarded((ws_bytes,), torch.uint8)
    assert ws.view.data_ptr() % 256 == 0   # torch allocations are 512-byte aligned, GUARD is a multiple of 256
    out = {"Y": Guarded((M, N), dt), "Z": Guarded((M, N), dt), "mean": Guarded((M,), torch.float32),
           "rstd": Guarded((M,), torch.float32)}
    api.fdl_forward(cfg.dtype, X, W, b, gamma, beta, cfg.eps, out["Y"].view, out["Z"].view, out["mean"].view,
                    out["rstd"].view, ws.view, stream=stream)
    if backward:
        dY = t["dY"].to(dev, dt)
        out.update({"dX": Guarded((M, K), dt), "dW": Guarded((N, K), dt), "db": Guarded((N,), torch.float32),
                    "dgamma": Guarded((N,), torch.float32), "dbeta": Guarded((N,), torch.float32)})
        api.fdl_backward(cfg.dtype, dY, X, W, gamma, out["Z"].view, out["mean"].view, out["rstd"].view,
                         out["dX"].view, out["dW"].view, out["db"].view, out["dgamma"].view, out["dbeta"].view,
                         ws.view, stream=stream)
    torch.cuda.synchronize()
    if check_guards:
        for k, g in out.items():
            assert g.intact(), f"kernel wrote outside the {k} buffer"
        assert ws.intact(), "kernel wrote outside the workspace"
    return {k: g.view for k, g in out.items()}


def to_f64(x: torch.Tensor) -> np.ndarray:
    return x.detach().to("cpu", torch.float32).numpy().astype(np.float64)


def check_f32(name: str, got: np.ndarray, ref: np.ndarray, rtol=1e-4, atol=1e-5):
    """fp32 bar: element-wise |got - ref| <= atol + rtol |ref| for every element."""
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{name}: non-finite output"
    if got.size == 0:
        return
    err = np.abs(got - ref)
    bad = err > atol + rtol * np.abs(ref)
    nbad = int(bad.sum())
    if nbad:
        i = np.unravel_index(np.argmax(err - (atol + rtol * np.abs(ref))), err.shape)
        raise AssertionError(f"{name}: {nbad}/{bad.size} elements outside atol={atol} rtol={rtol}; worst at {i}: "
                             f"got {got[i]!r} ref {ref[i]!r} err {err[i]:.3e}")


# every bf16 comparison leaves its achieved ratio here: (label, tensor name, ratio); tests that track the margin
# inside the bar read it back (see test_fullsize_gpu.py)
RATIO_LOG = []
_ratio_label = [""]


def set_ratio_label(label: str):
    _ratio_label[0] = label


def check_bf16(name: str, got: np.ndarray, ref: np.ndarray, bound=2e-2, zero_ref_atol=1e-3):
    """bf16 bar: max|got - ref| / max|ref| <= bound, per tensor.  Where the reference tensor is identically
    zero (degenerate rows: N = 1 or constant rows make Ahat = 0) the ratio is undefined and the absolute
    error must stay below `zero_ref_atol` instead.  Returns the achieved ratio and logs it."""
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{name}: non-finite output"
    if got.size == 0:
        return 0.0
    scale = np.abs(ref).max()
    err = np.abs(got - ref).max()
    if scale < 1e-9:
        assert err <= zero_ref_atol, f"{name}: reference is zero but max error is {err}"
        return 0.0
    ratio = err / scale
    RATIO_LOG.append((_ratio_label[0], name, float(ratio)))
    assert ratio <= bound, f"{name}: max|err|/max|ref| = {ratio:.3e} > {bound} (max err {err:.3e}, max ref {scale:.3e})"
    return ratio


U_BF16 = 2.0 ** -8     # relative spacing of bf16 (8 significant bits)


def backward_term_scale(n, ref, eps):
    """Sum of the magnitudes of the terms that make up each backward output (oracle-side, fp64): the scale against
    which rounding of the stored pre-activation and of the row statistics perturbs dZ = r (g - c1 - Ahat c2) GELU'(Z)
    when the three terms cancel (LayerNorm over one or two elements leaves a residue of order eps/var of them).
    Returns S for dX, dW, db, from S_dZ = r (|g| + |c1| + |Ahat c2|) (|GELU'(Z)| + 1e-4): the bf16 path evaluates
    Phi to an absolute (not relative) accuracy of 2.7e-5, so far in the left tail, where GELU' underflows, the
    rounding residue of the bracket meets a factor of that size rather than the true one."""
    from oracle import fdl_oracle as O
    Z, mean, rstd = ref["Z"], ref["mean"], ref["rstd"]
    A = O.gelu(Z)
    Ahat = (A - mean[:, None]) * rstd[:, None]
    g = n["dY"] * n["gamma"][None, :]
    c1 = g.mean(axis=1)
    c2 = (g * Ahat).mean(axis=1)
    S_dZ = rstd[:, None] * (np.abs(g) + np.abs(c1)[:, None] + np.abs(Ahat * c2[:, None])) * (np.abs(O.gelu_grad(Z)) + 1e-4)
    return {"dX": S_dZ @ np.abs(n["W"]), "dW": S_dZ.T @ np.abs(n["X"]), "db": S_dZ.sum(axis=0)}


def check_bf16_cancelling(name: str, got: np.ndarray, ref: np.ndarray, S: np.ndarray, bound=2e-2, c=2.0):
    """bf16 bar for outputs that are cancellation residues (LayerNorm rows of one or two elements): every element
    within bound * max|ref| + c * u_bf16 * S, S = sum of the magnitudes of the cancelling terms."""
    assert got.shape == ref.shape == S.shape, (name, got.shape, ref.shape, S.shape)
    assert np.all(np.isfinite(got)), f"{name}: non-finite output"
    tol = bound * np.abs(ref).max() + c * U_BF16 * S
    err = np.abs(got - ref)
    bad = err > tol
    if bad.any():
        i = np.unravel_index(np.argmax(err - tol), err.shape)
        raise AssertionError(f"{name}: {int(bad.sum())}/{bad.size} elements outside the condition-aware bound; worst at {i}: "
                             f"got {got[i]!r} ref {ref[i]!r} err {err[i]:.3e} tol {tol[i]:.3e}")


def check(cfg_dtype: str, name: str, got, ref, f32_atol=1e-5):
    if cfg_dtype == "f32":
        check_f32(name, got, ref, atol=f32_atol)
    else:
        check_bf16(name, got, ref)


OUTPUTS = ("Y", "dX", "dW", "db", "dgamma", "dbeta")
