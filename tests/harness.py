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


def check_bf16(name: str, got: np.ndarray, ref: np.ndarray, bound=2e-2, zero_ref_atol=1e-3):
    """bf16 bar: max|got - ref| / max|ref| <= bound, per tensor.  Where the reference tensor is identically
    zero (degenerate rows: N = 1 or constant rows make Ahat = 0) the ratio is undefined and the absolute
    error must stay below `zero_ref_atol` instead."""
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
    assert ratio <= bound, f"{name}: max|err|/max|ref| = {ratio:.3e} > {bound} (max err {err:.3e}, max ref {scale:.3e})"
    return ratio


def check(cfg_dtype: str, name: str, got, ref, f32_atol=1e-5):
    if cfg_dtype == "f32":
        check_f32(name, got, ref, atol=f32_atol)
    else:
        check_bf16(name, got, ref)


OUTPUTS = ("Y", "dX", "dW", "db", "dgamma", "dbeta")
