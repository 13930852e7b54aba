"""Pins of the oracle's options (CPU only): CosFace margin, the PFC* filter and the diagnostics.

arXiv 2203.15565: Sec. 4.1 (margin-based softmax with the hyper-parameters of CosFace and ArcFace),
Sec. 3.3 and Fig. 4 caption (PFC*: negatives whose cosine exceeds a fixed threshold, 0.4, are
filtered), Sec. 3.3 (definitions of APCS and AMNCS).
"""
import math

import numpy as np
import pytest
import torch

from oracle import pfc_oracle as O


def _rand(B, D, k, seed, wscale=1.0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((B, D)), rng.standard_normal((k, D)) * wscale, rng.integers(0, k, size=B)


def test_cosface_matches_autograd():
    X, W, y = _rand(7, 12, 19, 1)
    s, m = 30.0, 0.35
    out = O.forward_backward(X, W, y, s, m, margin="cosface")
    Xt = torch.tensor(X, requires_grad=True)
    Wt = torch.tensor(W, requires_grad=True)
    c = torch.nn.functional.normalize(Xt, dim=1) @ torch.nn.functional.normalize(Wt, dim=1).T
    z = s * (c - m * torch.nn.functional.one_hot(torch.tensor(y), 19).double())
    loss = torch.nn.functional.cross_entropy(z, torch.tensor(y))
    loss.backward()
    assert abs(out["loss"] - loss.item()) < 1e-12 * abs(loss.item())
    np.testing.assert_allclose(out["dX"], Xt.grad.numpy(), rtol=1e-9, atol=1e-13)
    np.testing.assert_allclose(out["dW"], Wt.grad.numpy(), rtol=1e-9, atol=1e-13)


def test_cosface_closed_form_and_m_zero():
    x = np.array([[1.0, 2.0, -0.5]])
    W = np.array([[0.3, 1.0, 0.2], [-1.0, 0.4, 0.9]])
    s, m = 16.0, 0.35
    c = (x / np.linalg.norm(x)) @ (W / np.linalg.norm(W, axis=1, keepdims=True)).T
    exp = math.log1p(math.exp(s * (c[0, 1] - c[0, 0] + m)))
    assert abs(O.forward_backward(x, W, np.array([0]), s, m, margin="cosface")["loss"] - exp) < 1e-12
    X, Wm, y = _rand(5, 6, 9, 2)
    a = O.forward_backward(X, Wm, y, 20.0, 0.0, margin="cosface")
    b = O.forward_backward(X, Wm, y, 20.0, 0.0, margin="arcface")
    assert abs(a["loss"] - b["loss"]) < 1e-13 and np.allclose(a["dW"], b["dW"], rtol=1e-12, atol=1e-15)
    with pytest.raises(ValueError):
        O.forward_backward(X, Wm, y, 20.0, 0.1, margin="sphereface")


def test_filter_disabled_is_identity():
    X, W, y = _rand(6, 8, 15, 3)
    base = O.forward_backward(X, W, y, 64.0, 0.5)
    for thr in (1.0, 1.5):
        f = O.forward_backward(X, W, y, 64.0, 0.5, filter_threshold=thr)
        assert f["loss"] == base["loss"] and (f["dW"] == base["dW"]).all() and (f["dX"] == base["dX"]).all()
        assert f["keep"].all()


def _brute_loss(X, W, y, s, m, thr):
    """Independent restatement with Python loops: Eq. 1 over the kept centers of each sample."""
    B, k = X.shape[0], W.shape[0]
    total = 0.0
    for i in range(B):
        xn = X[i] / math.sqrt(float(X[i] @ X[i]))
        zs = []
        zlab = None
        for j in range(k):
            wn = W[j] / math.sqrt(float(W[j] @ W[j]))
            c = max(-1.0, min(1.0, float(xn @ wn)))
            if j == y[i]:
                zlab = s * math.cos(math.acos(c) + m)
                zs.append(zlab)
            elif not (c > thr):
                zs.append(s * c)
        total += math.log(sum(math.exp(z - zlab) for z in zs))
    return total / B


def test_filter_matches_brute_force_and_zero_gradient():
    X, W, y = _rand(6, 5, 14, 4)            # D = 5: cosines are spread widely, many exceed 0.4
    s, m, thr = 16.0, 0.3, 0.4
    out = O.forward_backward(X, W, y, s, m, filter_threshold=thr)
    masked = ~out["keep"]
    assert masked.any() and not masked[np.arange(6), y].any()      # the label is never filtered
    assert abs(out["loss"] - _brute_loss(X, W, y, s, m, thr)) < 1e-12 * max(1.0, abs(out["loss"]))
    assert (out["p"][masked] == 0).all() and (out["dc"][masked] == 0).all()
    np.testing.assert_allclose(out["p"].sum(axis=1), 1.0, rtol=1e-12)
    # a filtered pair contributes nothing: removing the center from that sample's row of a
    # hand-built gradient reproduces dWn
    dWn = np.zeros_like(W)
    for i in range(6):
        for j in range(14):
            dWn[j] += out["dc"][i, j] * out["xn"][i]
    np.testing.assert_allclose(out["dWn"], dWn, rtol=1e-12, atol=1e-15)
    # filtering lowers the loss (the denominator of Eq. 1 shrinks)
    assert out["loss"] <= O.forward_backward(X, W, y, s, m)["loss"]


def test_filter_finite_differences():
    X, W, y = _rand(4, 5, 9, 5)
    s, m, thr = 12.0, 0.3, 0.4
    out = O.forward_backward(X, W, y, s, m, filter_threshold=thr)
    assert np.abs(out["cos"] - thr).min() > 1e-3           # no cosine sits on the threshold
    g = np.zeros_like(W)
    for j in range(9):
        for d in range(5):
            h = 1e-6
            Wp, Wm = W.copy(), W.copy()
            Wp[j, d] += h
            Wm[j, d] -= h
            g[j, d] = (O.forward_backward(X, Wp, y, s, m, filter_threshold=thr)["loss"] -
                       O.forward_backward(X, Wm, y, s, m, filter_threshold=thr)["loss"]) / (2 * h)
    assert np.abs(g - out["dW"]).max() <= 2e-6 * np.abs(out["dW"]).max()


def test_diagnostics_brute_force():
    X, W, y = _rand(5, 7, 11, 6)
    out = O.forward_backward(X, W, y, 64.0, 0.5, filter_threshold=0.2)
    apcs, amncs = 0.0, 0.0
    for i in range(5):
        cs = [float(X[i] @ W[j]) / (np.linalg.norm(X[i]) * np.linalg.norm(W[j])) for j in range(11)]
        apcs += cs[y[i]]
        amncs += max(c for j, c in enumerate(cs) if j != y[i])
    assert abs(out["apcs"] - apcs / 5) < 1e-13 and abs(out["amncs"] - amncs / 5) < 1e-13
