"""Pins for the sibling operators' fp64 oracle: each function is fixed to something other than itself -
closed forms and invariants, central finite differences, the same operator through torch's float64 functional ops
(and autograd for the backward pass), element-by-element Python loops on tiny shapes, and planted mistakes in copies
of the steps, which the pins must catch."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import siblings_oracle as S


def rnd(seed, *shape, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


T = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))


# ------------------------------------------------------------------ Linear + ReLU
def test_linear_relu_forward_by_hand_and_by_loops():
    X = np.array([[1.0, 2.0], [-1.0, 0.5]]); W = np.array([[1.0, -1.0], [0.5, 0.5], [-2.0, 0.0]]); b = np.array([0.5, -2.0, 0.0])
    # row 0: [1-2+.5, .5+1-2, -2] = [-0.5, -0.5, -2] -> 0;  row 1: [-1-.5+.5, -.5+.25-2, 2] = [-1, -2.25, 2]
    np.testing.assert_allclose(S.linear_relu_forward(X, W, b)["Y"], [[0, 0, 0], [0, 0, 2.0]], atol=0)
    X, W, b = rnd(1, 5, 4), rnd(2, 3, 4), rnd(3, 3)
    Y = S.linear_relu_forward(X, W, b)["Y"]
    for i in range(5):
        for j in range(3):
            z = sum(X[i, k] * W[j, k] for k in range(4)) + b[j]
            assert abs(Y[i, j] - max(z, 0.0)) < 1e-14
    # planted in copies of the step: a dropped bias, and a clamp from above instead of below, must not pass
    assert np.abs(np.maximum(X @ W.T, 0.0) - Y).max() > 1e-3
    assert np.abs(np.minimum(X @ W.T + b, 0.0) - Y).max() > 1e-3


@pytest.mark.parametrize("shape", [(4, 3, 5), (7, 6, 2), (1, 1, 1), (9, 5, 8)])
def test_linear_relu_backward_against_torch_autograd_and_finite_differences(shape):
    M, K, N = shape
    X, W, b, dY = rnd(10, M, K), rnd(11, N, K), rnd(12, N, scale=0.3), rnd(13, M, N)
    got = S.linear_relu_backward(dY, X, W, b)
    tx, tw, tb = T(X).requires_grad_(), T(W).requires_grad_(), T(b).requires_grad_()
    F.relu(F.linear(tx, tw, tb)).backward(T(dY))
    np.testing.assert_allclose(got["dX"], tx.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(got["dW"], tw.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(got["db"], tb.grad.numpy(), rtol=1e-12, atol=1e-13)
    # central differences of L = sum(dY * Y) (the inputs are generic: no pre-activation sits within h of the kink)
    assert np.abs(got["Z"]).min() > 1e-4
    L = lambda X_, W_, b_: float((dY * S.linear_relu_forward(X_, W_, b_)["Y"]).sum())
    h = 1e-6
    for name, arr, grad in (("dX", X, got["dX"]), ("dW", W, got["dW"]), ("db", b, got["db"])):
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            p, m = arr.copy(), arr.copy(); p[i] += h; m[i] -= h
            args_p = {"dX": (p, W, b), "dW": (X, p, b), "db": (X, W, p)}[name]
            args_m = {"dX": (m, W, b), "dW": (X, m, b), "db": (X, W, m)}[name]
            fd = (L(*args_p) - L(*args_m)) / (2 * h)
            assert abs(fd - grad[i]) < 1e-7 * max(1.0, abs(grad[i])), (name, i)


def test_linear_relu_backward_mask_conventions_and_planted_mistakes():
    X = np.array([[1.0, 1.0]]); W = np.array([[1.0, -1.0], [1.0, 1.0], [-1.0, -1.0]]); b = np.zeros(3)   # Z = [0, 2, -2]
    dY = np.array([[5.0, 7.0, 11.0]])
    g = S.linear_relu_backward(dY, X, W, b)
    np.testing.assert_array_equal(g["G"], [[0.0, 7.0, 0.0]])         # derivative at exactly 0 is 0; negative side 0
    np.testing.assert_array_equal(g["db"], [0.0, 7.0, 0.0])
    np.testing.assert_array_equal(g["dX"], [[7.0, 7.0]])
    np.testing.assert_array_equal(g["dW"], [[0, 0], [7.0, 7.0], [0, 0]])
    # planted mistakes in a copy: mask from Z >= 0, and unmasked gradient
    X, W, b, dY = rnd(20, 6, 4), rnd(21, 5, 4), rnd(22, 5), rnd(23, 6, 5)
    ref = S.linear_relu_backward(dY, X, W, b)
    Z = X @ W.T + b
    unmasked = dY @ W
    assert np.abs(unmasked - ref["dX"]).max() > 1e-2
    flipped = (dY * (Z < 0)) @ W
    assert np.abs(flipped - ref["dX"]).max() > 1e-2
    # linear in dY
    np.testing.assert_allclose(S.linear_relu_backward(2 * dY, X, W, b)["dW"], 2 * ref["dW"], rtol=1e-14)


# ------------------------------------------------------------------ LayerNorm forward
@pytest.mark.parametrize("shape", [(3, 7), (5, 64), (2, 1), (4, 2)])
def test_layernorm_forward_invariants_and_torch(shape):
    M, N = shape
    A, gamma, beta = rnd(30, M, N, scale=3.0) + 1.5, 1 + 0.3 * rnd(31, N), 0.3 * rnd(32, N)
    eps = 1e-5
    o = S.layernorm_forward(A, gamma, beta, eps)
    ref = F.layer_norm(T(A), (N,), T(gamma), T(beta), eps).numpy()
    np.testing.assert_allclose(o["Y"], ref, rtol=1e-12, atol=1e-12)
    Ahat = S.layernorm_forward(A, np.ones(N), np.zeros(N), eps)["Y"]
    np.testing.assert_allclose(Ahat.sum(axis=1), 0.0, atol=1e-11 * N)
    var = A.var(axis=1)                                         # numpy's own biased variance
    np.testing.assert_allclose((Ahat ** 2).mean(axis=1), var / (var + eps), rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(o["mean"], A.mean(axis=1), rtol=1e-13)
    # with eps -> 0 the normalised rows have variance exactly 1 (N > 1)
    if N > 1:
        np.testing.assert_allclose((S.layernorm_forward(A, np.ones(N), np.zeros(N), 0.0)["Y"] ** 2).mean(axis=1), 1.0, rtol=1e-12)
    # planted: unbiased variance, eps outside the root
    mu = A.mean(axis=1, keepdims=True)
    if N > 1:
        unb = (A - mu) / np.sqrt(A.var(axis=1, ddof=1, keepdims=True) + eps) * gamma + beta
        assert np.abs(unb - ref).max() > 1e-4
    out = (A - mu) / (np.sqrt(A.var(axis=1, keepdims=True)) + eps) * gamma + beta
    if N > 1:
        assert np.abs(out - ref).max() > 1e-8


def test_layernorm_constant_row_and_loops():
    A = np.full((2, 5), 3.25); gamma = np.arange(1.0, 6.0); beta = np.arange(5.0) * 0.1
    np.testing.assert_allclose(S.layernorm_forward(A, gamma, beta)["Y"], np.broadcast_to(beta, (2, 5)), atol=1e-12)
    A = rnd(33, 3, 4)
    Y = S.layernorm_forward(A, gamma[:4], beta[:4], 1e-3)["Y"]
    for i in range(3):
        m = sum(A[i]) / 4
        v = sum((a - m) ** 2 for a in A[i]) / 4
        for j in range(4):
            assert abs(Y[i, j] - ((A[i, j] - m) / math.sqrt(v + 1e-3) * gamma[j] + beta[j])) < 1e-14


# ------------------------------------------------------------------ RMSNorm forward
@pytest.mark.parametrize("shape", [(3, 7), (5, 64), (2, 1)])
def test_rmsnorm_forward_invariants_and_torch(shape):
    M, N = shape
    A, w = rnd(40, M, N, scale=2.0) + 0.7, 1 + 0.3 * rnd(41, N)
    eps = 1e-5
    o = S.rmsnorm_forward(A, w, eps)
    ref = F.rms_norm(T(A), (N,), T(w), eps).numpy()
    np.testing.assert_allclose(o["Y"], ref, rtol=1e-12, atol=1e-13)
    ms = (A ** 2).mean(axis=1)
    np.testing.assert_allclose(((o["Y"] / w) ** 2).mean(axis=1), ms / (ms + eps), rtol=1e-12)
    # scale invariance at eps = 0, and no mean subtraction (a constant row maps to sign * weight)
    np.testing.assert_allclose(S.rmsnorm_forward(7.5 * A, w, 0.0)["Y"], S.rmsnorm_forward(A, w, 0.0)["Y"], rtol=1e-12)
    np.testing.assert_allclose(S.rmsnorm_forward(np.full((1, N), -2.0), w, 0.0)["Y"], -w[None, :], rtol=1e-13)
    # loops
    for i in range(M):
        r = 1.0 / math.sqrt(sum(a * a for a in A[i]) / N + eps)
        for j in range(N):
            assert abs(o["Y"][i, j] - A[i, j] * r * w[j]) < 1e-13 * max(1.0, abs(o["Y"][i, j]))
    # planted: a mean-subtracting (LayerNorm-like) variant must differ
    lnlike = (A - A.mean(axis=1, keepdims=True)) / np.sqrt(A.var(axis=1, keepdims=True) + eps) * w
    if N > 1:
        assert np.abs(lnlike - ref).max() > 1e-3


# ------------------------------------------------------------------ SiLU and the Llama feed-forward block
def test_silu_closed_forms():
    assert S.silu(0.0) == 0.0
    z = np.linspace(-30, 30, 241)
    np.testing.assert_allclose(S.silu(z) - S.silu(-z), z, rtol=1e-13, atol=1e-13)   # sigmoid(z) + sigmoid(-z) = 1
    np.testing.assert_allclose(S.silu(z), F.silu(T(z)).numpy(), rtol=1e-13, atol=1e-15)
    assert abs(S.silu(40.0) - 40.0) < 1e-12 and abs(S.silu(-40.0)) < 1e-15
    assert abs(S.silu(1.0) - 1.0 / (1.0 + math.exp(-1.0))) < 1e-16
    # minimum of z sigmoid(z) is at z = -1.27846454..., value -0.27846454...
    zz = np.linspace(-1.3, -1.25, 5001)
    assert abs(zz[np.argmin(S.silu(zz))] + 1.2784645) < 2e-5 and abs(S.silu(zz).min() + 0.2784645) < 1e-7


@pytest.mark.parametrize("shape", [(3, 4, 6), (5, 8, 2), (1, 1, 1), (6, 5, 9)])
def test_llama_ffn_forward_against_torch_and_loops(shape):
    M, D, H = shape
    X, Wg, Wu, Wd = rnd(50, M, D), rnd(51, H, D) / math.sqrt(D), rnd(52, H, D) / math.sqrt(D), rnd(53, D, H) / math.sqrt(H)
    o = S.llama_ffn_forward(X, Wg, Wu, Wd)
    tx = T(X)
    ref = F.linear(F.silu(F.linear(tx, T(Wg))) * F.linear(tx, T(Wu)), T(Wd)).numpy()
    np.testing.assert_allclose(o["Y"], ref, rtol=1e-12, atol=1e-13)
    for i in range(M):
        for d in range(D):
            acc = 0.0
            for h in range(H):
                g = sum(X[i, k] * Wg[h, k] for k in range(D)); u = sum(X[i, k] * Wu[h, k] for k in range(D))
                acc += g / (1.0 + math.exp(-g)) * u * Wd[d, h]
            assert abs(acc - o["Y"][i, d]) < 1e-12 * max(1.0, abs(acc))
    if H > 1 and D > 1:
        # planted: gate and up exchanged; a transposed down projection is a shape error unless D == H
        swapped = S.llama_ffn_forward(X, Wu, Wg, Wd)["Y"]
        assert np.abs(swapped - ref).max() > 1e-4
    # zero gate weights: SiLU(0) = 0 annihilates the block
    assert np.abs(S.llama_ffn_forward(X, np.zeros_like(Wg), Wu, Wd)["Y"]).max() == 0.0
