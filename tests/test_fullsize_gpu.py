"""GPU parity at the full sizes of the large seeded configurations, in the launch configuration the benchmark
times (same entry points, same workspace sizing, same kernels).

cfg3 (16384 x 4096 x 4096, shifted X) and cfg4 (65536 x 2048 x 8192, the benchmark's workload, with the dense dY the
benchmark times): the oracle does the whole thing, streamed over row blocks - dW, db, dgamma, dbeta, mean, rstd are
compared in full, Y, dX and Zsave on sampled rows (they are local to a row given W).
Additional property cases (cfg4 and a tall ragged batch): dY zero outside a sampled set S of rows - then dZ is exactly
zero outside S, so the sums over rows run over S alone and the oracle computes them from those rows, while the HIP path
still runs the full-size launch; and dX must be exactly zero on every other row.

Every bf16 comparison's achieved max|err|/max|ref| is logged; for the seeded configurations it must also stay within
twice the level recorded below, so that a drift inside the 2e-2 bar is seen.
"""
import sys

import numpy as np
import pytest
import torch

from oracle import fdl_oracle as O
from paper_2509_14279_amd import inputs as I
import harness as H

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


# Error levels of the HIP path on the seeded bf16 configurations, max|err|/max|ref| per tensor against the whole
# fp64 oracle, as recorded on an MI355X when these tests were written (they are error levels, not expected output
# values: the outputs themselves are only ever compared with the oracle).  A run must stay within twice each level.
RECORDED_RATIO = {
    ("cfg1_bf16_8192x1024x4096", "dW"): 3.605e-03,
    ("cfg1_bf16_8192x1024x4096", "db"): 5.914e-04,
    ("cfg1_bf16_8192x1024x4096", "dgamma"): 2.464e-03,
    ("cfg1_bf16_8192x1024x4096", "dbeta"): 4.482e-08,
    ("cfg1_bf16_8192x1024x4096", "mean"): 2.277e-04,
    ("cfg1_bf16_8192x1024x4096", "Y[rows]"): 4.619e-03,
    ("cfg1_bf16_8192x1024x4096", "dX[rows]"): 3.428e-03,
    ("cfg1_bf16_8192x1024x4096", "Zsave[rows]"): 2.813e-03,
    ("cfg3_bf16_16384x4096x4096_shifted", "dW"): 3.541e-03,
    ("cfg3_bf16_16384x4096x4096_shifted", "db"): 1.046e-04,
    ("cfg3_bf16_16384x4096x4096_shifted", "dgamma"): 1.947e-03,
    ("cfg3_bf16_16384x4096x4096_shifted", "dbeta"): 3.427e-08,
    ("cfg3_bf16_16384x4096x4096_shifted", "mean"): 1.693e-04,
    ("cfg3_bf16_16384x4096x4096_shifted", "Y[rows]"): 3.611e-03,
    ("cfg3_bf16_16384x4096x4096_shifted", "dX[rows]"): 3.226e-03,
    ("cfg3_bf16_16384x4096x4096_shifted", "Zsave[rows]"): 3.242e-03,
    ("cfg4_bf16_65536x2048x8192", "dW"): 3.532e-03,
    ("cfg4_bf16_65536x2048x8192", "db"): 5.560e-04,
    ("cfg4_bf16_65536x2048x8192", "dgamma"): 2.203e-03,
    ("cfg4_bf16_65536x2048x8192", "dbeta"): 3.839e-08,
    ("cfg4_bf16_65536x2048x8192", "mean"): 2.087e-04,
    ("cfg4_bf16_65536x2048x8192", "Y[rows]"): 4.540e-03,
    ("cfg4_bf16_65536x2048x8192", "dX[rows]"): 3.362e-03,
    ("cfg4_bf16_65536x2048x8192", "Zsave[rows]"): 3.139e-03,
}


def check_ratio_drift(label):
    seen = {name: r for (lab, name, r) in H.RATIO_LOG if lab == label}
    say("[ratios] " + label + ": " + ", ".join(f"{k}={v:.3e}" for k, v in seen.items()))
    for name, r in seen.items():
        rec = RECORDED_RATIO.get((label, name))
        if rec is not None:
            assert r <= 2.0 * rec + 1e-6, f"{label} {name}: max|err|/max|ref| = {r:.3e}, recorded level {rec:.3e}"


def whole_oracle_check(cfg, n_rows, block_rows):
    """The HIP path on the seeded inputs with the dense dY against the whole streamed oracle."""
    say(f"[fullsize] {cfg.name}: generating inputs")
    t = I.generate(cfg)
    say(f"[fullsize] {cfg.name}: running HIP path")
    got = H.run_fdl(cfg, t, check_guards=True)
    n = {k: v.numpy() for k, v in t.items()}
    rows = np.random.default_rng(cfg.seed).choice(cfg.M, size=n_rows, replace=False)
    say(f"[fullsize] {cfg.name}: running oracle over all {cfg.M} rows (streamed)")
    ref = O.forward_backward_streamed(n["X"], n["W"], n["b"], n["gamma"], n["beta"], n["dY"], cfg.eps,
                                      block_rows=block_rows, keep_rows=rows)
    H.set_ratio_label(cfg.name)
    for k in ("dW", "db", "dgamma", "dbeta", "mean"):
        H.check_bf16(k, H.to_f64(got[k]), ref[k])
    np.testing.assert_allclose(H.to_f64(got["rstd"]), ref["rstd"], rtol=2e-2)
    kr = ref["kept_rows"]
    idx = torch.as_tensor(kr, device="cuda")
    H.check_bf16("Y[rows]", H.to_f64(got["Y"][idx]), ref["kept_Y"])
    H.check_bf16("dX[rows]", H.to_f64(got["dX"][idx]), ref["kept_dX"])
    H.check_bf16("Zsave[rows]", H.to_f64(got["Z"][idx]), ref["kept_Z"])
    # anti-shortcut: outputs of the full-size run are not degenerate
    ysamp = H.to_f64(got["Y"][idx])
    # (a column whose gamma happens to round to zero is constant, so the column test is on all but a few)
    assert ysamp.std(axis=1).min() > 0.1 and (ysamp.std(axis=0) > 0.01).mean() > 0.99
    check_ratio_drift(cfg.name)


def test_cfg1_bf16_mid_ratios():
    whole_oracle_check(I.CONFIGS[1], n_rows=8192, block_rows=2048)


def test_cfg3_bf16_shifted_full():
    whole_oracle_check(I.CONFIGS[3], n_rows=96, block_rows=2048)


def test_cfg4_bf16_headline_dense_full():
    whole_oracle_check(I.CONFIGS[4], n_rows=64, block_rows=1024)


def sampled_check(cfg, extra_rows=()):
    """Sampled outputs one by one, and full sums over rows through a row-sparse dY (see the module docstring)."""
    H.set_ratio_label(cfg.name + "/sampled")
    say(f"[fullsize] {cfg.name}: generating inputs")
    t = I.generate(cfg)
    rng = np.random.default_rng(4)
    rows = np.unique(np.concatenate([rng.choice(cfg.M, size=64, replace=False), np.asarray(extra_rows, dtype=np.int64)]))
    say(f"[fullsize] {cfg.name}: HIP path, dense dY")
    got = H.run_fdl(cfg, t, check_guards=True)
    n = {k: v.numpy() for k, v in t.items()}
    say(f"[fullsize] {cfg.name}: oracle on {len(rows)} sampled rows")
    ref = O.forward_backward_streamed(n["X"], n["W"], n["b"], n["gamma"], n["beta"], n["dY"], cfg.eps,
                                      block_rows=64, rows=rows, keep_rows=rows)
    idx = torch.as_tensor(ref["kept_rows"], device="cuda")
    H.check_bf16("Y[rows]", H.to_f64(got["Y"][idx]), ref["kept_Y"])
    H.check_bf16("dX[rows]", H.to_f64(got["dX"][idx]), ref["kept_dX"])
    H.check_bf16("Zsave[rows]", H.to_f64(got["Z"][idx]), ref["kept_Z"])
    H.check_bf16("mean[rows]", H.to_f64(got["mean"][idx]), ref["mean"][ref["kept_rows"]])
    np.testing.assert_allclose(H.to_f64(got["rstd"][idx]), ref["rstd"][ref["kept_rows"]], rtol=2e-2)
    dbeta_ref = n["dY"].sum(axis=0, dtype=np.float64)
    H.check_bf16("dbeta", H.to_f64(got["dbeta"]), dbeta_ref)
    # anti-shortcut: outputs of the full-size run are not degenerate
    ysamp = H.to_f64(got["Y"][idx])
    # (a column whose gamma happens to round to zero is constant, so the column test is on all but a few)
    assert ysamp.std(axis=1).min() > 0.1 and (ysamp.std(axis=0) > 0.01).mean() > 0.99
    del got

    # ---- dY supported on a sampled set of rows: the sums over rows are computable in full
    S = np.unique(np.concatenate([rng.choice(cfg.M, size=256, replace=False), np.asarray(extra_rows, dtype=np.int64)]))
    dY_sparse = torch.zeros_like(t["dY"])
    dY_sparse[torch.as_tensor(S)] = t["dY"][torch.as_tensor(S)]
    t2 = dict(t)
    t2["dY"] = dY_sparse
    say(f"[fullsize] {cfg.name}: HIP path, dY supported on {len(S)} rows")
    got = H.run_fdl(cfg, t2, check_guards=True)
    say(f"[fullsize] {cfg.name}: oracle over those rows")
    ref = O.forward_backward_streamed(n["X"], n["W"], n["b"], n["gamma"], n["beta"], dY_sparse.numpy(), cfg.eps,
                                      block_rows=64, rows=S, keep_rows=S)
    for k in ("dW", "db", "dgamma", "dbeta"):
        H.check_bf16(k, H.to_f64(got[k]), ref[k])
    idx = torch.as_tensor(ref["kept_rows"], device="cuda")
    H.check_bf16("dX[S]", H.to_f64(got["dX"][idx]), ref["kept_dX"])
    mask = torch.ones(cfg.M, dtype=torch.bool, device="cuda")
    mask[idx] = False
    assert float(got["dX"][mask].float().abs().max()) == 0.0, "rows with zero upstream gradient must have dX = 0"


def test_cfg4_bf16_headline_sampled():
    sampled_check(I.CONFIGS[4])


def test_tall_ragged_batch_bf16_sampled():
    """More than 2^31 bytes per M x N tensor (64-bit offsets everywhere) and a ragged row count on the fast path:
    partial last row tile in F1 and dX, dW as fast kernel over the first rows plus the generic kernel over the last 64."""
    M = (1 << 20) + 64
    sampled_check(I.custom("bf16", M, 128, 2048, seed=37), extra_rows=(0, M - 1, M - 64, M - 65, (1 << 20) - 1))
