"""Pins for the fp64 oracle: each test fixes it to something other than itself.

What the mathematics fixes:
  * Phi, phi: a 40-digit Taylor/series evaluation in decimal arithmetic;
    GELU(0)=0, GELU'(0)=1/2, GELU(z)-GELU(-z)=z, GELU'(z)+GELU'(-z)=1.
  * LayerNorm rows: mean 0 and mean square var/(var+eps) before the affine
    step (exactly 1 as eps -> 0).
  * Its gradient: sum_j dA = 0 and sum_j dA*Ahat = r N c2 eps/(var+eps).
  * All five gradients: central finite differences of L = sum(dY * Y).
  * The composed operator through torch's float64 functional ops + autograd
    (a different library route: F.gelu / F.layer_norm kernels and reverse-mode
    differentiation instead of hand-derived formulas).
  * Element-by-element Python loops on tiny shapes (math.erfc, no numpy).
  * Degenerate cases: N = 1, W = 0, rows made constant, M=N=K=1.
  * Planted mistakes in copies of the oracle's steps must be caught.
"""
import math
from decimal import Decimal, getcontext

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import fdl_oracle as O

RNG = np.random.default_rng(12345)


def tiny(M, K, N, seed=0, scale_x=1.0):
    r = np.random.default_rng(seed)
    return dict(
        X=r.standard_normal((M, K)) * scale_x,
        W=r.standard_normal((N, K)) / math.sqrt(K),
        b=r.standard_normal(N) * 0.3,
        gamma=1.0 + 0.3 * r.standard_normal(N),
        beta=0.3 * r.standard_normal(N),
        dY=r.standard_normal((M, N)),
    )


# ------------------------------------------------------------------ Phi, phi
def _erf_series(x: Decimal) -> Decimal:
    """erf(x) = 2/sqrt(pi) * sum_n (-1)^n x^(2n+1) / (n! (2n+1)), 60 digits."""
    getcontext().prec = 60
    term = x
    total = x
    n = 0
    x2 = x * x
    while True:
        n += 1
        term = -term * x2 / n
        add = term / (2 * n + 1)
        total += add
        if abs(add) < Decimal(10) ** -55:
            break
    pi = Decimal("3.14159265358979323846264338327950288419716939937510582097494")
    return 2 * total / pi.sqrt()


@pytest.mark.parametrize("z", [-4.0, -2.5, -1.0, -0.3, 0.0, 0.5, 1.0, 1.96, 3.0, 4.5])
def test_Phi_phi_against_decimal_series(z):
    getcontext().prec = 60
    zd = Decimal(repr(z))
    Phi_ref = (1 + _erf_series(zd / Decimal(2).sqrt())) / 2
    pi = Decimal("3.14159265358979323846264338327950288419716939937510582097494")
    phi_ref = (-(zd * zd) / 2).exp() / (2 * pi).sqrt()
    assert float(O.Phi(z)) == pytest.approx(float(Phi_ref), rel=2e-15, abs=1e-300)
    assert float(O.phi(z)) == pytest.approx(float(phi_ref), rel=2e-15)
    assert float(O.gelu(z)) == pytest.approx(float(zd * Phi_ref), rel=4e-15, abs=1e-300)
    assert float(O.gelu_grad(z)) == pytest.approx(float(Phi_ref + zd * phi_ref), rel=1e-14, abs=1e-18)


def test_gelu_closed_forms():
    assert float(O.gelu(0.0)) == 0.0
    assert float(O.gelu_grad(0.0)) == 0.5
    z = np.linspace(-8, 8, 1601)
    np.testing.assert_allclose(O.gelu(z) - O.gelu(-z), z, rtol=0, atol=4e-16 * 8)
    np.testing.assert_allclose(O.gelu_grad(z) + O.gelu_grad(-z), 1.0, rtol=0, atol=1e-15)
    # tails: GELU -> z, GELU' -> 1 on the right; both -> 0 (from below / above) on the left
    assert float(O.gelu(40.0)) == 40.0 and float(O.gelu_grad(40.0)) == 1.0
    assert -1e-300 < float(O.gelu(-40.0)) <= 0.0
    assert abs(float(O.gelu_grad(-40.0))) < 1e-300
    # minimum of GELU near z = -0.7518 with value about -0.17
    zz = np.linspace(-1.5, 0, 150001)
    i = np.argmin(O.gelu(zz))
    assert abs(zz[i] - (-0.75179)) < 1e-4 and abs(O.gelu(zz[i]) - (-0.169964)) < 1e-5
    assert abs(float(O.gelu_grad(zz[i]))) < 2e-5


# --------------------------------------------------------- forward invariants
@pytest.mark.parametrize("shape", [(7, 5, 33), (16, 64, 128), (3, 2, 2)])
def test_layernorm_row_invariants(shape):
    t = tiny(*shape, seed=3)
    eps = 1e-5
    f = O.forward(t["X"], t["W"], t["b"], np.ones(shape[2]), np.zeros(shape[2]), eps)
    Ahat = f["Y"]                                   # gamma = 1, beta = 0
    A = O.gelu(f["Z"])
    var = A.var(axis=1)                             # numpy's biased variance
    np.testing.assert_allclose(Ahat.mean(axis=1), 0.0, atol=1e-13)
    np.testing.assert_allclose((Ahat ** 2).mean(axis=1), var / (var + eps), rtol=1e-12)
    np.testing.assert_allclose(f["mean"], A.mean(axis=1), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(f["rstd"], 1 / np.sqrt(var + eps), rtol=1e-13)
    # eps -> 0: variance exactly one
    f0 = O.forward(t["X"], t["W"], t["b"], np.ones(shape[2]), np.zeros(shape[2]), 0.0)
    np.testing.assert_allclose((f0["Y"] ** 2).mean(axis=1), 1.0, rtol=1e-12)
    # affine step is per column
    f2 = O.forward(t["X"], t["W"], t["b"], t["gamma"], t["beta"], eps)
    np.testing.assert_allclose(f2["Y"], Ahat * t["gamma"][None] + t["beta"][None], rtol=1e-14, atol=1e-15)


def test_linear_step_by_hand():
    X = np.array([[1.0, 2.0, 3.0], [-1.0, 0.5, 4.0]])
    W = np.array([[1.0, 0.0, -1.0], [2.0, 1.0, 0.0], [0.5, 0.5, 0.5], [0.0, -3.0, 1.0]])   # [N=4,K=3]
    b = np.array([0.1, -0.2, 0.3, 0.0])
    Z = O.linear(X, W, b)
    hand = np.array([[1 - 3 + 0.1, 2 + 2 - 0.2, 3.0 + 0.3, -6 + 3.0],
                     [-1 - 4 + 0.1, -2 + 0.5 - 0.2, 1.75 + 0.3, -1.5 + 4.0]])
    np.testing.assert_allclose(Z, hand, rtol=0, atol=1e-15)


def test_zero_weight_makes_rows_identical():
    t = tiny(6, 4, 9, seed=5)
    f = O.forward(t["X"], np.zeros_like(t["W"]), t["b"], t["gamma"], t["beta"])
    np.testing.assert_array_equal(f["Z"], np.broadcast_to(t["b"], f["Z"].shape))
    assert np.all(f["Y"] == f["Y"][0])
    # and that row is LayerNorm(GELU(b)) computed by hand
    A = np.array([bj * 0.5 * math.erfc(-bj / math.sqrt(2)) for bj in t["b"]])
    mu = A.sum() / 9
    var = ((A - mu) ** 2).sum() / 9
    np.testing.assert_allclose(f["Y"][0], (A - mu) / math.sqrt(var + 1e-5) * t["gamma"] + t["beta"], rtol=1e-13)


def test_degenerate_rows():
    # N = 1: A - mu = 0 so Ahat = 0, Y = beta; every gradient but dbeta vanishes
    t = tiny(5, 3, 1, seed=7)
    r = O.forward_backward(t["X"], t["W"], t["b"], t["gamma"], t["beta"], t["dY"])
    np.testing.assert_array_equal(r["Y"], np.broadcast_to(t["beta"], (5, 1)))
    np.testing.assert_allclose(r["rstd"], 1 / math.sqrt(1e-5), rtol=1e-15)
    for k in ("dX", "dW", "db", "dgamma"):
        assert np.all(r[k] == 0.0), k
    np.testing.assert_allclose(r["dbeta"], t["dY"].sum(axis=0), rtol=1e-15)
    # scalar case M=N=K=1 is the same statement
    r1 = O.forward_backward([[2.0]], [[3.0]], [0.5], [1.5], [-0.25], [[7.0]])
    assert r1["Y"].item() == -0.25 and r1["Z"].item() == 6.5 and r1["dbeta"].item() == 7.0
    assert r1["dX"].item() == 0.0 and r1["dW"].item() == 0.0
    # constant row (W = 0, b constant): variance 0, eps keeps r finite, Y = beta
    f = O.forward(np.ones((2, 3)), np.zeros((4, 3)), np.full(4, 0.7), np.ones(4) * 2, np.arange(4.0))
    np.testing.assert_allclose(f["Y"], np.broadcast_to(np.arange(4.0), (2, 4)), atol=1e-12)
    assert np.all(np.isfinite(f["rstd"]))


# -------------------------------------------------------- backward invariants
def test_layernorm_backward_row_invariants():
    t = tiny(9, 6, 40, seed=11)
    eps = 1e-5
    f = O.forward(t["X"], t["W"], t["b"], t["gamma"], t["beta"], eps)
    rows = O.backward_rows(t["dY"], t["gamma"], f["Z"], f["mean"], f["rstd"])
    dA = rows["dZ"] / O.gelu_grad(f["Z"])
    Ahat = rows["Ahat"]
    N = 40
    var = O.gelu(f["Z"]).var(axis=1)
    c2 = (t["dY"] * t["gamma"][None] * Ahat).mean(axis=1)
    np.testing.assert_allclose(dA.sum(axis=1), 0.0, atol=1e-12)
    np.testing.assert_allclose((dA * Ahat).sum(axis=1), f["rstd"] * N * c2 * eps / (var + eps), rtol=1e-6, atol=1e-12)


def test_backward_linear_in_dY_and_dbeta_is_column_sum():
    t = tiny(8, 5, 12, seed=13)
    r1 = O.forward_backward(t["X"], t["W"], t["b"], t["gamma"], t["beta"], t["dY"])
    r2 = O.forward_backward(t["X"], t["W"], t["b"], t["gamma"], t["beta"], 2.0 * t["dY"])
    for k in ("dX", "dW", "db", "dgamma", "dbeta"):
        np.testing.assert_allclose(r2[k], 2.0 * r1[k], rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(r1["dbeta"], t["dY"].sum(axis=0), rtol=1e-15)
    # rows with dY = 0 contribute nothing: restricting to the other rows is exact
    dY = t["dY"].copy()
    dY[[1, 4, 5]] = 0.0
    full = O.forward_backward(t["X"], t["W"], t["b"], t["gamma"], t["beta"], dY)
    sub = O.forward_backward_streamed(t["X"], t["W"], t["b"], t["gamma"], t["beta"], dY,
                                      block_rows=2, rows=[0, 2, 3, 6, 7])
    for k in ("dW", "db", "dgamma", "dbeta"):
        np.testing.assert_allclose(sub[k], full[k], rtol=1e-13, atol=1e-14)
    assert np.all(full["dX"][[1, 4, 5]] == 0.0)


# --------------------------------------------------------- finite differences
def _loss(t, dY, eps):
    return float((dY * O.forward(t["X"], t["W"], t["b"], t["gamma"], t["beta"], eps)["Y"]).sum())


@pytest.mark.parametrize("shape,seed", [((1, 1, 2), 0), ((2, 3, 4), 1), ((3, 5, 2), 2), ((5, 4, 5), 3), ((4, 2, 7), 4)])
def test_all_gradients_by_central_differences(shape, seed):
    t = tiny(*shape, seed=seed)
    eps = 1e-5
    an = O.forward_backward(t["X"], t["W"], t["b"], t["gamma"], t["beta"], t["dY"], eps)
    h = 1e-6
    for name, gname in (("X", "dX"), ("W", "dW"), ("b", "db"), ("gamma", "dgamma"), ("beta", "dbeta")):
        num = np.zeros_like(t[name])
        it = np.nditer(t[name], flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = t[name][idx]
            t[name][idx] = old + h
            lp = _loss(t, t["dY"], eps)
            t[name][idx] = old - h
            lm = _loss(t, t["dY"], eps)
            t[name][idx] = old
            num[idx] = (lp - lm) / (2 * h)
        scale = max(1.0, np.abs(an[gname]).max())
        np.testing.assert_allclose(an[gname], num, rtol=0, atol=2e-7 * scale, err_msg=gname)


# ------------------------------------------------------ torch float64 autograd
@pytest.mark.parametrize("shape,seed", [((5, 3, 4), 0), ((33, 17, 65), 1), ((128, 96, 200), 2), ((64, 256, 512), 3)])
def test_against_torch_float64_autograd(shape, seed):
    t = tiny(*shape, seed=seed, scale_x=1.0 if seed != 3 else 30.0)
    eps = 1e-5
    tt = {k: torch.tensor(v, dtype=torch.float64, requires_grad=(k != "dY")) for k, v in t.items()}
    N = shape[2]
    Y = F.layer_norm(F.gelu(F.linear(tt["X"], tt["W"], tt["b"]), approximate="none"), (N,), tt["gamma"], tt["beta"], eps)
    Y.backward(tt["dY"])
    r = O.forward_backward(t["X"], t["W"], t["b"], t["gamma"], t["beta"], t["dY"], eps)
    np.testing.assert_allclose(r["Y"], Y.detach().numpy(), rtol=1e-10, atol=1e-12)
    for name, gname in (("X", "dX"), ("W", "dW"), ("b", "db"), ("gamma", "dgamma"), ("beta", "dbeta")):
        ref = tt[name].grad.numpy()
        np.testing.assert_allclose(r[gname], ref, rtol=1e-9, atol=1e-11 * max(1.0, np.abs(ref).max()), err_msg=gname)


# ------------------------------------------------------------ plain loops
def _loops(X, W, b, gamma, beta, dY, eps):
    """The operator and its gradient element by element, Python floats only."""
    M, K, N = len(X), len(X[0]), len(W)
    s2, s2pi = math.sqrt(2.0), math.sqrt(2.0 * math.pi)
    Y = [[0.0] * N for _ in range(M)]
    dX = [[0.0] * K for _ in range(M)]
    dW = [[0.0] * K for _ in range(N)]
    db, dg, dbt = [0.0] * N, [0.0] * N, [0.0] * N
    for i in range(M):
        z = [sum(X[i][k] * W[j][k] for k in range(K)) + b[j] for j in range(N)]
        a = [zj * 0.5 * math.erfc(-zj / s2) for zj in z]
        mu = sum(a) / N
        var = sum((aj - mu) ** 2 for aj in a) / N
        r = 1.0 / math.sqrt(var + eps)
        ah = [(aj - mu) * r for aj in a]
        for j in range(N):
            Y[i][j] = ah[j] * gamma[j] + beta[j]
        g = [dY[i][j] * gamma[j] for j in range(N)]
        c1 = sum(g) / N
        c2 = sum(g[j] * ah[j] for j in range(N)) / N
        for j in range(N):
            dA = r * (g[j] - c1 - ah[j] * c2)
            gp = 0.5 * math.erfc(-z[j] / s2) + z[j] * math.exp(-0.5 * z[j] * z[j]) / s2pi
            dz = dA * gp
            db[j] += dz
            dg[j] += dY[i][j] * ah[j]
            dbt[j] += dY[i][j]
            for k in range(K):
                dX[i][k] += dz * W[j][k]
                dW[j][k] += dz * X[i][k]
    return dict(Y=Y, dX=dX, dW=dW, db=db, dgamma=dg, dbeta=dbt)


@pytest.mark.parametrize("shape,seed", [((2, 3, 4), 21), ((5, 2, 3), 22), ((4, 7, 6), 23)])
def test_against_python_loops(shape, seed):
    t = tiny(*shape, seed=seed)
    ref = _loops(*(t[k].tolist() for k in ("X", "W", "b", "gamma", "beta", "dY")), 1e-5)
    r = O.forward_backward(t["X"], t["W"], t["b"], t["gamma"], t["beta"], t["dY"], 1e-5)
    for k in ("Y", "dX", "dW", "db", "dgamma", "dbeta"):
        np.testing.assert_allclose(r[k], np.array(ref[k]), rtol=1e-12, atol=1e-13, err_msg=k)


def test_streamed_equals_whole():
    t = tiny(37, 9, 21, seed=31)
    whole = O.forward_backward(t["X"], t["W"], t["b"], t["gamma"], t["beta"], t["dY"])
    st = O.forward_backward_streamed(t["X"], t["W"], t["b"], t["gamma"], t["beta"], t["dY"],
                                     block_rows=8, keep_rows=[0, 13, 36])
    for k in ("dW", "db", "dgamma", "dbeta", "mean", "rstd"):
        np.testing.assert_allclose(st[k], whole[k], rtol=1e-13, atol=1e-14, err_msg=k)
    for k in ("Y", "Z", "dX"):
        np.testing.assert_allclose(st["kept_" + k], whole[k][st["kept_rows"]], rtol=1e-13, atol=1e-14)


# ------------------------------------------------------- planted mistakes
def _fd_dX(fwd, t, eps=1e-5, h=1e-6):
    num = np.zeros_like(t["X"])
    for idx in np.ndindex(*t["X"].shape):
        old = t["X"][idx]
        t["X"][idx] = old + h
        lp = float((t["dY"] * fwd(t)).sum())
        t["X"][idx] = old - h
        lm = float((t["dY"] * fwd(t)).sum())
        t["X"][idx] = old
        num[idx] = (lp - lm) / (2 * h)
    return num


@pytest.mark.parametrize("mistake", ["drop_c1", "drop_c2", "sign_phi", "transpose_W", "unbiased_var", "eps_outside"])
def test_planted_mistakes_are_caught(mistake, monkeypatch):
    """Each plausible slip, planted into the oracle on the CPU, must break a pin."""
    t = tiny(4, 4, 4, seed=41)      # square so a transposed operand still has a valid shape
    eps = 1e-2                      # large enough that misplacing eps is visible

    def run():
        return O.forward_backward(t["X"], t["W"], t["b"], t["gamma"], t["beta"], t["dY"], eps)

    good = run()
    if mistake == "drop_c1":
        orig = O.backward_rows

        def bad(dY, gamma, Z, mean, rstd):
            o = orig(dY, gamma, Z, mean, rstd)
            g = np.asarray(dY) * np.asarray(gamma)[None]
            o["dZ"] = o["dZ"] + (rstd[:, None] * g.mean(axis=1)[:, None]) * O.gelu_grad(Z)
            return o
        monkeypatch.setattr(O, "backward_rows", bad)
    elif mistake == "drop_c2":
        orig = O.backward_rows

        def bad(dY, gamma, Z, mean, rstd):
            o = orig(dY, gamma, Z, mean, rstd)
            g = np.asarray(dY) * np.asarray(gamma)[None]
            c2 = (g * o["Ahat"]).mean(axis=1)
            o["dZ"] = o["dZ"] + (rstd[:, None] * o["Ahat"] * c2[:, None]) * O.gelu_grad(Z)
            return o
        monkeypatch.setattr(O, "backward_rows", bad)
    elif mistake == "sign_phi":
        monkeypatch.setattr(O, "gelu_grad", lambda z: O.Phi(z) - np.asarray(z) * O.phi(z))
    elif mistake == "transpose_W":
        monkeypatch.setattr(O, "linear", lambda X, W, b: np.asarray(X) @ np.asarray(W) + np.asarray(b)[None])
    elif mistake == "unbiased_var":
        def bad_stats(A, eps_):
            mu = A.mean(axis=1)
            var = A.var(axis=1, ddof=1)
            return mu, var, 1 / np.sqrt(var + eps_)
        monkeypatch.setattr(O, "row_stats", bad_stats)
    elif mistake == "eps_outside":
        def bad_stats(A, eps_):
            mu = A.mean(axis=1)
            var = A.var(axis=1)
            return mu, var, 1 / (np.sqrt(var) + eps_)
        monkeypatch.setattr(O, "row_stats", bad_stats)
    bad_r = run()

    # pin 1: torch float64 route for Y and dX
    tt = {k: torch.tensor(v, dtype=torch.float64, requires_grad=(k != "dY")) for k, v in t.items()}
    Y = F.layer_norm(F.gelu(F.linear(tt["X"], tt["W"], tt["b"])), (4,), tt["gamma"], tt["beta"], eps)
    Y.backward(tt["dY"])
    ok_good = np.allclose(good["Y"], Y.detach().numpy(), rtol=1e-10, atol=1e-12) and \
        np.allclose(good["dX"], tt["X"].grad.numpy(), rtol=1e-9, atol=1e-11)
    ok_bad = np.allclose(bad_r["Y"], Y.detach().numpy(), rtol=1e-10, atol=1e-12) and \
        np.allclose(bad_r["dX"], tt["X"].grad.numpy(), rtol=1e-9, atol=1e-11)
    assert ok_good and not ok_bad

    # pin 2: finite differences of the (possibly broken) forward against its own backward
    # catch backward-only slips without any library in the loop.
    if mistake in ("drop_c1", "drop_c2", "sign_phi"):
        num = _fd_dX(lambda tt_: O.forward(tt_["X"], tt_["W"], tt_["b"], tt_["gamma"], tt_["beta"], eps)["Y"], t, eps)
        assert not np.allclose(bad_r["dX"], num, rtol=0, atol=1e-6)
        assert np.allclose(good["dX"], num, rtol=0, atol=1e-6)
