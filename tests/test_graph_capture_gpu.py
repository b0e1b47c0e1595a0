"""The forward and backward entry points under HIP graph capture: they allocate nothing, clear memory with kernels
rather than memsets, and enqueue everything on the stream they are given, so a captured graph of one training step
must replay to the same bits as the eager calls - several replays, with eager work and synchronisation between them.
(The first, eager call also does the once-per-kernel set-up that is not capturable.)"""
import pytest
import torch

from paper_2509_14279_amd import api, inputs as I

pytestmark = pytest.mark.gpu

OUT = ("Y", "Z", "mean", "rstd", "dX", "dW", "db", "dg", "dbt")


def _buffers(cfg, t):
    dt = I.storage_torch_dtype(cfg.dtype)
    dev = "cuda"
    M, K, N = cfg.M, cfg.K, cfg.N
    b = {k: t[k].to(dev, dt) for k in ("X", "W", "dY")}
    b.update({k: t[k].to(dev) for k in ("b", "gamma", "beta")})
    b.update(Y=torch.empty(M, N, device=dev, dtype=dt), Z=torch.empty(M, N, device=dev, dtype=dt),
             mean=torch.empty(M, device=dev), rstd=torch.empty(M, device=dev),
             dX=torch.empty(M, K, device=dev, dtype=dt), dW=torch.empty(N, K, device=dev, dtype=dt),
             db=torch.empty(N, device=dev), dg=torch.empty(N, device=dev), dbt=torch.empty(N, device=dev),
             ws=torch.empty(api.fdl_workspace_bytes(cfg.dtype, M, K, N), dtype=torch.uint8, device=dev))
    return b


def _step(cfg, b, stream):
    api.fdl_forward(cfg.dtype, b["X"], b["W"], b["b"], b["gamma"], b["beta"], cfg.eps, b["Y"], b["Z"], b["mean"], b["rstd"],
                    b["ws"], stream)
    api.fdl_backward(cfg.dtype, b["dY"], b["X"], b["W"], b["gamma"], b["Z"], b["mean"], b["rstd"], b["dX"], b["dW"], b["db"],
                     b["dg"], b["dbt"], b["ws"], stream)


@pytest.mark.parametrize("dtype,shape", [("bf16", (2048, 1024, 2048)),    # paired dX + dW launch, finishing launch, blocked dZ
                                         ("bf16", (1000, 256, 768)),      # ragged batch: padded tail copy, generic dW tail
                                         ("bf16", (300, 200, 264)),       # padded mode: weight copies, zeroed dZ columns
                                         ("f32", (130, 70, 200))])        # generic kernels, partial statistics
def test_one_step_replays_from_a_graph(dtype, shape):
    M, K, N = shape
    cfg = I.custom(dtype, M, K, N, seed=900 + M)
    t = I.generate(cfg)
    b = _buffers(cfg, t)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        _step(cfg, b, side)                       # eager reference (and one-time kernel set-up)
    side.synchronize()
    ref = {k: b[k].clone() for k in OUT}
    for k in OUT:
        b[k].fill_(7.0)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        _step(cfg, b, side)
    for replay in range(3):
        for k in OUT:
            b[k].fill_(-3.0)                      # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in OUT:
            assert torch.equal(b[k].view(torch.uint8), ref[k].view(torch.uint8)), (cfg.name, k, replay)
