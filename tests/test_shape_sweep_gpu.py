"""Shape-generalisation sweep: the whole block against the oracle over a grid of shapes the kernels were not tuned
on, with several seeds and several input distributions per shape (many inputs x many initialisations, in the
spirit of the paper's robust benchmark settings: its section on the robust kernel benchmark and the evaluation
appendix).  Small enough for the fp64 oracle to do every case whole."""
import sys

import numpy as np
import pytest

from oracle import fdl_oracle as O
from paper_2509_14279_amd import inputs as I
import harness as H

pytestmark = pytest.mark.gpu

# (M, K, N): around every switch of the launch plan - tile edges of the generic GEMM (16/64/128), the fast path's
# 256-alignment, vector width (N % 8, N % 4), the row-resident kernels' widths (512 x 2^k, 8192) and the
# reduction-length granularity of the fast pipeline (128).
GRID = [
    (3, 5, 7), (16, 16, 16), (65, 17, 33), (127, 129, 255), (128, 128, 128), (129, 127, 513), (255, 64, 1025),
    (256, 128, 256), (256, 192, 512), (256, 256, 1536), (512, 128, 4608), (257, 128, 256), (256, 128, 264),
    (512, 384, 768), (768, 256, 2048), (40, 300, 4104), (9, 2, 8192), (12, 40, 8208), (1024, 128, 256), (33, 1, 1),
]
# input distributions: (x_mean, x_std)
INITS = [(0.0, 1.0), (3.0, 0.2), (-1.0, 5.0)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("init", range(len(INITS)))
@pytest.mark.parametrize("shape", GRID)
def test_shape_seed_init_grid(shape, init, dtype):
    M, K, N = shape
    x_mean, x_std = INITS[init]
    for seed in (7000 + 13 * init + M + K + N, 9000 + 17 * init + M * 3 + N):
        cfg = I.custom(dtype, M, K, N, seed=seed, x_mean=x_mean, x_std=x_std)
        print(f"[sweep] {cfg.name} init={init}", flush=True)
        sys.stdout.flush()
        t = I.generate(cfg)
        got = H.run_fdl(cfg, t)
        n = {k: v.numpy().astype(np.float64) for k, v in t.items()}
        ref = O.forward_backward(n["X"], n["W"], n["b"], n["gamma"], n["beta"], n["dY"], cfg.eps)
        outputs = H.OUTPUTS
        if dtype == "bf16" and N <= 2:
            outputs = ("Y", "dbeta", "dgamma")      # LayerNorm over <= 2 elements: the rest is cancellation residue
        f32_atol = 1e-3 if N == 1 else 1e-5         # N = 1: rstd = eps^-1/2 multiplies the fp32 rounding of the mean
        H.set_ratio_label(cfg.name)
        for k in outputs:
            H.check(cfg.dtype, k, H.to_f64(got[k]), ref[k], f32_atol=1e-5 if k == "dbeta" else f32_atol)
        if len(outputs) < len(H.OUTPUTS):
            # the residues are held to the condition-aware bound: bar + 2 u_bf16 x magnitude of the cancelling terms
            S = H.backward_term_scale(n, ref, cfg.eps)
            for k in ("dX", "dW", "db"):
                H.check_bf16_cancelling(k, H.to_f64(got[k]), ref[k], S[k])
