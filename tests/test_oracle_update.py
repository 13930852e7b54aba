"""Pins of the oracle's sparse SGD-momentum update and of the whole step (CPU only).

arXiv 2203.15565: Eq. 3 (center update), abstract and text after Eq. 4 (all centers are kept,
only the sampled ones are updated in an iteration).
"""
import numpy as np
import torch

from oracle import pfc_oracle as O


def _state(N, D, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((N, D)) * 0.01, rng.standard_normal((N, D)) * 0.001


def test_unsampled_rows_bit_identical():
    W, v = _state(50, 8, 1)
    W0, v0 = W.copy(), v.copy()
    idx = np.array([3, 7, 20, 49], dtype=np.int32)
    g = np.random.default_rng(2).standard_normal((4, 8))
    O.update(W, v, idx, g, 0.1, 0.9)
    rest = np.setdiff1d(np.arange(50), idx)
    assert W[rest].tobytes() == W0[rest].tobytes()
    assert v[rest].tobytes() == v0[rest].tobytes()
    np.testing.assert_allclose(v[idx], 0.9 * v0[idx] + g, rtol=0, atol=0)
    np.testing.assert_allclose(W[idx], W0[idx] - 0.1 * (0.9 * v0[idx] + g), rtol=0, atol=0)


def test_lr_zero_and_mu_zero():
    W, v = _state(10, 4, 3)
    W0, v0 = W.copy(), v.copy()
    idx = np.array([1, 5])
    g = np.ones((2, 4))
    O.update(W, v, idx, g, 0.0, 0.9)
    assert (W == W0).all()
    assert (v[idx] == 0.9 * v0[idx] + g).all()
    W, v = W0.copy(), v0.copy()
    O.update(W, v, idx, g, 0.5, 0.0)
    assert (W[idx] == W0[idx] - 0.5 * g).all()
    assert (v[idx] == g).all()


def test_lazy_momentum():
    """A row skipped in an iteration keeps its momentum untouched: sampled at steps 1 and 3 only
    => v3 = mu*g1 + g3 (not mu^2*g1 + g3)."""
    W = np.zeros((6, 3))
    v = np.zeros((6, 3))
    g1, g2, g3 = np.full((1, 3), 1.0), np.full((1, 3), 10.0), np.full((1, 3), 100.0)
    O.update(W, v, np.array([2]), g1, 0.1, 0.9)
    O.update(W, v, np.array([4]), g2, 0.1, 0.9)      # row 2 not sampled
    O.update(W, v, np.array([2]), g3, 0.1, 0.9)
    assert np.allclose(v[2], 0.9 * 1.0 + 100.0)
    assert np.allclose(W[2], -0.1 * 1.0 - 0.1 * (0.9 + 100.0))
    # sampled twice in a row: v2 = mu*g1 + g2
    W[:] = 0
    v[:] = 0
    O.update(W, v, np.array([1]), g1, 0.1, 0.9)
    O.update(W, v, np.array([1]), g2, 0.1, 0.9)
    assert np.allclose(v[1], 0.9 + 10.0)


def test_r_one_equals_dense_torch_sgd():
    """At r = 1 every row is sampled and the step equals torch.optim.SGD(momentum) on the
    library-evaluated loss, over several iterations."""
    N, B, D = 30, 6, 8
    rng = np.random.default_rng(5)
    W0 = rng.standard_normal((N, D)) * 0.1
    s, m, lr, mu = 16.0, 0.0, 0.05, 0.9
    W, v = W0.copy(), np.zeros((N, D))
    Wt = torch.tensor(W0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([Wt], lr=lr, momentum=mu)
    for t in range(4):
        X = rng.standard_normal((B, D))
        y = rng.integers(0, N, size=B)
        loss, _, idx, _, _ = O.step(X, y, W, v, r=1.0, s=s, m=m, lr=lr, mu=mu, seed=0, step=t)
        opt.zero_grad()
        logits = s * torch.nn.functional.normalize(torch.tensor(X), dim=1) @ \
            torch.nn.functional.normalize(Wt, dim=1).T
        lt = torch.nn.functional.cross_entropy(logits, torch.tensor(y))
        lt.backward()
        opt.step()
        assert abs(loss - lt.item()) < 1e-10 * abs(lt.item())
        np.testing.assert_allclose(W, Wt.detach().numpy(), rtol=1e-9, atol=1e-13)


def test_step_touches_only_sampled_rows_and_replays():
    N, B, D = 200, 8, 8
    rng = np.random.default_rng(6)
    W0 = rng.standard_normal((N, D)) * 0.01
    v0 = rng.standard_normal((N, D)) * 0.001
    X = rng.standard_normal((B, D))
    y = rng.integers(0, N, size=B)
    W, v = W0.copy(), v0.copy()
    loss, dX, idx, yl, fb = O.step(X, y, W, v, r=0.1, s=64.0, m=0.5, lr=0.1, mu=0.9, seed=3, step=5)
    rest = np.setdiff1d(np.arange(N), idx)
    assert rest.size == N - 20
    assert W[rest].tobytes() == W0[rest].tobytes() and v[rest].tobytes() == v0[rest].tobytes()
    assert (W[idx] != W0[idx]).any(axis=1).all()
    # replay from the saved state with the same (seed, step): bit-identical
    W2, v2 = W0.copy(), v0.copy()
    loss2, dX2, idx2, _, _ = O.step(X, y, W2, v2, r=0.1, s=64.0, m=0.5, lr=0.1, mu=0.9, seed=3, step=5)
    assert loss2 == loss and (idx2 == idx).all() and W2.tobytes() == W.tobytes()
