"""Pins of the oracle's loss and gradients (CPU only).

Cited passages are of arXiv 2203.15565: Eq. 1 (softmax loss, mean over B), Eq. 2 / Eq. 4
(feature gradient, sum restricted to the sampled set), Eq. 3 (center gradient), Sec. 4.3
("loss of PFC is lower than the baseline as the denominator of Eq. 1 is smaller"), Tab. 1
(r = 1.0 is the full FC layer).
"""
import math

import numpy as np
import pytest
import torch

from oracle import pfc_oracle as O


def _rand(B, D, k, seed, wscale=0.01):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((B, D))
    W = rng.standard_normal((k, D)) * wscale
    y = rng.integers(0, k, size=B)
    return X, W, y


def test_m_zero_equals_library_cross_entropy():
    """m = 0: the loss is plain CE of s*cosine logits -- checked against torch's own routine."""
    X, W, y = _rand(9, 16, 23, 1)
    s = 64.0
    out = O.forward_backward(X, W, y, s, 0.0)
    Xt = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    logits = s * torch.nn.functional.normalize(Xt, dim=1) @ torch.nn.functional.normalize(Wt, dim=1).T
    loss = torch.nn.functional.cross_entropy(logits, torch.tensor(y))
    loss.backward()
    assert abs(out["loss"] - loss.item()) < 1e-12 * max(1.0, abs(loss.item()))
    np.testing.assert_allclose(out["dX"], Xt.grad.numpy(), rtol=1e-9, atol=1e-13)
    np.testing.assert_allclose(out["dW"], Wt.grad.numpy(), rtol=1e-9, atol=1e-13)


def test_arcface_matches_autograd_of_angle_form():
    """m > 0: compare with torch autograd on the independent form s*cos(acos(c) + m)."""
    X, W, y = _rand(7, 12, 19, 2, wscale=1.0)
    s, m = 30.0, 0.5
    out = O.forward_backward(X, W, y, s, m)
    Xt = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    c = torch.nn.functional.normalize(Xt, dim=1) @ torch.nn.functional.normalize(Wt, dim=1).T
    onehot = torch.nn.functional.one_hot(torch.tensor(y), W.shape[0]).bool()
    theta = torch.acos(c.clamp(-1 + 1e-15, 1 - 1e-15))
    z = s * torch.where(onehot, torch.cos(theta + m), c)
    loss = torch.nn.functional.cross_entropy(z, torch.tensor(y))
    loss.backward()
    assert abs(out["loss"] - loss.item()) < 1e-11 * abs(loss.item())
    np.testing.assert_allclose(out["dX"], Xt.grad.numpy(), rtol=1e-7, atol=1e-12)
    np.testing.assert_allclose(out["dW"], Wt.grad.numpy(), rtol=1e-7, atol=1e-12)


def test_closed_form_equal_centers():
    """All sampled centers equal and m = 0  =>  uniform softmax  =>  loss = ln k."""
    rng = np.random.default_rng(3)
    X = rng.standard_normal((5, 8))
    W = np.tile(rng.standard_normal((1, 8)), (11, 1))
    y = rng.integers(0, 11, size=5)
    out = O.forward_backward(X, W, y, 64.0, 0.0)
    assert abs(out["loss"] - math.log(11)) < 1e-12


def test_closed_form_two_classes():
    """B = 1, k = 2: loss = ln(1 + exp(s*(c2 - cos(theta1 + m))))."""
    x = np.array([[1.0, 2.0, -0.5]])
    W = np.array([[0.3, 1.0, 0.2], [-1.0, 0.4, 0.9]])
    s, m = 16.0, 0.35
    c = (x / np.linalg.norm(x)) @ (W / np.linalg.norm(W, axis=1, keepdims=True)).T
    exp = math.log1p(math.exp(s * (c[0, 1] - math.cos(math.acos(c[0, 0]) + m))))
    out = O.forward_backward(x, W, np.array([0]), s, m)
    assert abs(out["loss"] - exp) < 1e-12 * max(1.0, exp)


def test_scale_invariance():
    X, W, y = _rand(6, 10, 13, 4)
    base = O.forward_backward(X, W, y, 64.0, 0.5)
    X2 = X * np.linspace(0.1, 7.0, 6)[:, None]
    W2 = W * np.linspace(3.0, 0.2, 13)[:, None]
    out = O.forward_backward(X2, W2, y, 64.0, 0.5)
    assert abs(out["loss"] - base["loss"]) < 1e-10 * abs(base["loss"])
    np.testing.assert_allclose(out["dXn"], base["dXn"], rtol=1e-9, atol=1e-14)


def test_subset_lowers_loss():
    """Sec. 4.3: a smaller denominator in Eq. 1 gives a lower loss: S subset S' => L(S) <= L(S')."""
    X, W, y = _rand(8, 16, 40, 5, wscale=1.0)
    y = y % 10                                  # labels inside the first 10 rows
    full = O.forward_backward(X, W, y, 64.0, 0.5)["loss"]
    prev = -np.inf
    for k in (10, 17, 29, 40):
        cur = O.forward_backward(X, W[:k], y, 64.0, 0.5)["loss"]
        assert cur >= prev - 1e-12
        prev = cur
    assert abs(prev - full) < 1e-12


def test_r_one_is_full_fc():
    """PFC at r = 1 equals the margin softmax over all N classes (Tab. 1 rows 'FC-1.0')."""
    N, B, D = 37, 6, 8
    rng = np.random.default_rng(6)
    X = rng.standard_normal((B, D))
    W = rng.standard_normal((N, D))
    labels = rng.integers(0, N, size=B)
    idx, yl, k = O.sample(labels, N, 1.0, seed=0, step=0)
    a = O.forward_backward(X, W[idx], yl, 64.0, 0.5)
    b = O.forward_backward(X, W, labels, 64.0, 0.5)
    assert a["loss"] == b["loss"]
    assert (a["dW"] == b["dW"]).all()


@pytest.mark.parametrize("s,m,wscale", [(64.0, 0.5, 0.01), (8.0, 0.3, 1.0), (1.0, 0.0, 1.0)])
def test_finite_differences(s, m, wscale):
    """Central differences on every entry of X and of the sampled centers."""
    B, D, k = 4, 6, 7
    X, W, y = _rand(B, D, k, 7, wscale)
    y[0] = y[1]                                  # duplicate label
    out = O.forward_backward(X, W, y, s, m)

    def loss_at(Xa, Wa):
        return O.forward_backward(Xa, Wa, y, s, m)["loss"]

    gX = np.zeros_like(X)
    for i in range(B):
        for d in range(D):
            h = 1e-6 * max(1.0, abs(X[i, d]))
            Xp, Xm = X.copy(), X.copy()
            Xp[i, d] += h
            Xm[i, d] -= h
            gX[i, d] = (loss_at(Xp, W) - loss_at(Xm, W)) / (2 * h)
    gW = np.zeros_like(W)
    for j in range(k):
        for d in range(D):
            h = 1e-6 * max(wscale, abs(W[j, d]))
            Wp, Wm = W.copy(), W.copy()
            Wp[j, d] += h
            Wm[j, d] -= h
            gW[j, d] = (loss_at(X, Wp) - loss_at(X, Wm)) / (2 * h)
    scale_x = np.abs(out["dX"]).max()
    scale_w = np.abs(out["dW"]).max()
    assert np.abs(gX - out["dX"]).max() <= 2e-6 * scale_x
    assert np.abs(gW - out["dW"]).max() <= 2e-6 * scale_w


def test_gradient_invariants():
    X, W, y = _rand(8, 16, 21, 8)
    s, m = 64.0, 0.5
    o = O.forward_backward(X, W, y, s, m)
    B = X.shape[0]
    # probabilities sum to one; dz rows sum to zero
    np.testing.assert_allclose(o["p"].sum(axis=1), 1.0, rtol=1e-12)
    dz = o["p"].copy()
    dz[np.arange(B), y] -= 1
    assert np.abs(dz.sum(axis=1)).max() < 1e-12
    # raw-row gradients are tangent to the sphere
    assert np.abs((o["dX"] * X).sum(axis=1)).max() < 1e-12 * np.abs(o["dX"]).max() * np.abs(X).max() * 16
    assert np.abs((o["dW"] * W).sum(axis=1)).max() < 1e-12 * np.abs(o["dW"]).max() * np.abs(W).max() * 16
    # t_j and u_i are the column / row sums of dc*c
    np.testing.assert_allclose(o["t"], (o["dc"] * o["cos"]).sum(axis=0), rtol=1e-9, atol=1e-15)
    np.testing.assert_allclose(o["u"], (o["dc"] * o["cos"]).sum(axis=1), rtol=1e-9, atol=1e-15)
    # a class that is nobody's label gets (s/B) * sum_i p_ij * projected xn_i / |W_j|
    j = next(j for j in range(21) if j not in set(y.tolist()))
    g = (s / B) * (o["p"][:, j][:, None] * o["xn"]).sum(axis=0)
    g = (g - (g @ o["wn"][j]) * o["wn"][j]) / o["w_norm"][j]
    np.testing.assert_allclose(o["dW"][j], g, rtol=1e-9, atol=1e-16)


def test_eq4_recovered_without_scale_margin_norm():
    """s = 1, m = 0, unit-norm inputs: B*dXn_i = -((1-p+)W+ - sum_{j in S, j != y} p_j W_j)  (Eq. 4),
    and B*dWn_j = -(sum_{i in B+}(1-p_i)x_i - sum_{i in B-} p_i x_i)  (bracket of Eq. 3)."""
    X, W, y = _rand(5, 9, 12, 9, wscale=1.0)
    X /= np.linalg.norm(X, axis=1, keepdims=True)
    W /= np.linalg.norm(W, axis=1, keepdims=True)
    o = O.forward_backward(X, W, y, 1.0, 0.0)
    B = X.shape[0]
    logits = X @ W.T
    p = np.exp(logits) / np.exp(logits).sum(axis=1, keepdims=True)
    for i in range(B):
        g = -(1 - p[i, y[i]]) * W[y[i]]
        for j in range(12):
            if j != y[i]:
                g = g + p[i, j] * W[j]
        np.testing.assert_allclose(B * o["dXn"][i], g, rtol=1e-10, atol=1e-14)
    for j in range(12):
        g = np.zeros(9)
        for i in range(B):
            g += (-(1 - p[i, j]) if y[i] == j else p[i, j]) * X[i]
        np.testing.assert_allclose(B * o["dWn"][j], g, rtol=1e-10, atol=1e-14)


def test_rejects_bad_label():
    X, W, y = _rand(3, 4, 5, 10)
    y[0] = 5
    with pytest.raises(ValueError):
        O.forward_backward(X, W, y, 64.0, 0.5)
