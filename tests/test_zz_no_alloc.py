"""fdl_forward_static (the forward pass on the library's own fixed scratch array, for callers that cannot allocate)
against fdl_forward on the same inputs: same kernels on a different scratch address, so every output must agree bit
for bit (stricter than the parity bars, which the fdl_forward side is held to against the oracle elsewhere) - except
where the array is too small for the transposed weights that fdl_forward uses for large batches (own test below).

Two calls in a row on one GPU, the second with a smaller input, through shapes whose forward pass really uses the
scratch: partial row statistics from the GEMM epilogue (rows longer than the row-resident normalisation holds, and the
generic kernel), and the padded copy of X's last rows (ragged M on the bf16 fast path).  This file is collected
last, so that a failure here cannot hide the other tests."""
import sys

import pytest
import torch

from paper_2509_14279_amd import api, inputs as I

pytestmark = pytest.mark.gpu

FWD_OUT = ("Y", "Z", "mean", "rstd")


def run_forward(cfg, t, static: bool):
    dt = I.storage_torch_dtype(cfg.dtype)
    dev = "cuda"
    M, K, N = cfg.M, cfg.K, cfg.N
    X = t["X"].to(dev, dt); W = t["W"].to(dev, dt)
    b = t["b"].to(dev); gamma = t["gamma"].to(dev); beta = t["beta"].to(dev)
    # outputs start from a fill that no result can equal by accident, so a location the call skipped is caught
    out = {"Y": torch.full((M, N), 7.0, device=dev, dtype=dt), "Z": torch.full((M, N), 7.0, device=dev, dtype=dt),
           "mean": torch.full((M,), 7.0, device=dev), "rstd": torch.full((M,), -7.0, device=dev)}
    if static:
        api.fdl_forward_static(cfg.dtype, X, W, b, gamma, beta, cfg.eps, out["Y"], out["Z"], out["mean"], out["rstd"])
    else:
        ws = torch.empty(api.fdl_workspace_bytes(cfg.dtype, M, K, N), dtype=torch.uint8, device=dev)
        api.fdl_forward(cfg.dtype, X, W, b, gamma, beta, cfg.eps, out["Y"], out["Z"], out["mean"], out["rstd"], ws)
    torch.cuda.synchronize()
    return out


def test_forward_static_matches_forward_on_two_calls_in_a_row():
    # first the larger problem, then smaller ones that reuse (part of) the same scratch bytes
    cases = [I.custom("bf16", 385, 512, 8448, seed=51),     # fast path, ragged M (padded X tail) + epilogue partials
             I.custom("f32", 130, 70, 200, seed=52),        # generic kernel partials, smaller
             I.custom("bf16", 300, 256, 512, seed=53),      # fast path, ragged M, row-resident normalisation
             I.custom("bf16", 200, 136, 264, seed=54),      # padded mode: zero-padded weight copy + X tail in the scratch
             I.custom("bf16", 16384, 128, 256, seed=55)]    # large batch: transposed weights in the scratch
    inputs = [I.generate(c, with_dY=False) for c in cases]
    got = []
    for c, t in zip(cases, inputs):                          # the static calls back to back, nothing in between
        print(f"[no-alloc] static {c.name}", flush=True)
        sys.stdout.flush()
        got.append(run_forward(c, t, static=True))
    for c, t, g in zip(cases, inputs, got):
        print(f"[no-alloc] workspace {c.name}", flush=True)
        ref = run_forward(c, t, static=False)
        for k in FWD_OUT:
            assert torch.equal(g[k].view(torch.uint8), ref[k].view(torch.uint8)), (c.name, k)
            assert torch.isfinite(g[k].float()).all(), (c.name, k)


def test_forward_static_with_weights_too_large_to_transpose_in_the_array():
    # a large batch: fdl_forward transposes W into its workspace (2 N K = 17.8 MB here); the array has no room for that,
    # so the static entry point runs the same contraction on W as it is.  Different kernels: compared to the parity
    # bar of bf16 storage rather than bit for bit.
    c = I.custom("bf16", 32768, 2048, 4352, seed=56)
    assert 2 * c.N * c.K > api.FDL_STATIC_SCRATCH_BYTES
    t = I.generate(c, with_dY=False)
    got = run_forward(c, t, static=True)
    ref = run_forward(c, t, static=False)
    for k in FWD_OUT:
        g, r = got[k].float(), ref[k].float()
        assert torch.isfinite(g).all(), k
        assert (g - r).abs().max().item() <= 2e-2 * r.abs().max().item(), k


def test_forward_static_rejects_what_the_array_cannot_hold():
    dev = "cuda"
    # 8 bytes per (row, 64-column tile): 32768 x 128 tiles = 32 MiB of partial statistics > 16 MiB
    M, K, N = 32768, 8, 8192
    z = torch.zeros(16, device=dev)
    st = api.fdl_forward_static_raw("f32", M, K, N, z, z, z, z, z, 1e-5, z, z, z, z, None)
    assert st == api.FDL_ERR_WORKSPACE
    assert api.fdl_workspace_bytes("f32", M, K, N) > api.FDL_STATIC_SCRATCH_BYTES
