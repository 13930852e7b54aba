"""Plain fp64 CPU oracle of one Partial FC (PFC) training step.

TEST INFRASTRUCTURE ONLY.  This module is the slow, obviously-correct statement of what
the HIP library must compute.  It shares no code, table or constant with the GPU path and
is imported only by tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py.

What it follows (arXiv 2203.15565, "Partial FC"):
  * Sec. 3.2, first paragraph and Fig. 4 caption: every class that occurs in the batch
    (a "positive" center) goes into the buffer first, random negative centers fill the
    rest; |S| = C*r (text after Eq. 4).  Sec. 3.3: the smallest ratio keeps only the
    within-batch classes.
  * Eq. 1: softmax cross entropy, mean over the batch, evaluated over the sampled set S
    only (Eq. 4 restricts the sum to j in S).  The paper trains with the margin-based
    variant (Sec. 4.1, "hyper-parameters of margin-based softmax loss"); the formula is
    not printed there, so the ArcFace form  s*cos(theta + m)  on the label logit is the
    default; the CosFace form  s*(cos(theta) - m)  is the option.  Sec. 3.3 / Fig. 4 caption:
    the PFC* variant filters negatives above a fixed cosine threshold; Sec. 3.3 defines the
    diagnostics APCS and AMNCS.
  * Eq. 2 / Eq. 4: gradient w.r.t. the feature; Eq. 3: gradient / update of a center.
    They are printed for the plain soft-max; here they are carried through the scale,
    the margin and the two L2 normalisations by the chain rule.
  * Sec. 3.2, text after Eq. 4: only the sampled centers are updated in an iteration.

Readings fixed where the paper is silent (all of them are listed in the design notes):
  k = max(U, ceil(r*N)), r*N evaluated in binary64; negatives are the top scores of an
  i.i.d. Philox4x32-10 score per class, ties to the smaller class id; the buffer is kept
  in ascending class id; both x and W rows are L2-normalised (eps 1e-12); cosines are
  clamped to [-1, 1]; no easy-margin / fallback branch for theta + m > pi; SGD with
  momentum (dampening 0, no Nesterov, no weight decay) and *lazy* momentum: rows outside
  S keep W and v bit for bit.

Parity status: every function below is pinned by tests/test_oracle_*.py (Philox
known-answer vectors, brute-force selection, set invariants, library cross entropy at
m = 0, closed forms, finite differences, dense torch SGD at r = 1).  The composition of the
pieces into one step has no printed value in the paper: whole-step parity is pinned only
through that decomposition.
"""
from __future__ import annotations

import math

import numpy as np

__all__ = [
    "philox4x32_10",
    "class_scores",
    "num_sampled",
    "sample",
    "forward_backward",
    "update",
    "step",
]

_M32 = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)
# Philox4x32 round multipliers and Weyl key increments (Salmon et al., SC'11, Sec. 3.3 / Tab. 2).
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = np.uint64(0x9E3779B9)
_PHILOX_W1 = np.uint64(0xBB67AE85)

EPS_NORM = 1e-12   # lower bound on a row norm before dividing
EPS_SIN2 = 1e-12   # lower bound on 1 - c^2 inside the margin derivative


def philox4x32_10(counter, key):
    """Philox4x32 with 10 rounds (Salmon et al., SC'11).

    counter: 4 arrays (or scalars) of 32-bit words, key: 2 words.  Returns 4 uint64 arrays
    holding 32-bit words.  All arithmetic is done in uint64 so the 32x32 -> 64 bit products
    are exact.
    """
    c0, c1, c2, c3 = [np.asarray(c, dtype=np.uint64) & _M32 for c in counter]
    k0, k1 = [np.asarray(k, dtype=np.uint64) & _M32 for k in key]
    for _ in range(10):
        p0 = _PHILOX_M0 * c0
        p1 = _PHILOX_M1 * c2
        c0, c1, c2, c3 = (
            (p1 >> _S32) ^ c1 ^ k0,
            p1 & _M32,
            (p0 >> _S32) ^ c3 ^ k1,
            p0 & _M32,
        )
        k0 = (k0 + _PHILOX_W0) & _M32
        k1 = (k1 + _PHILOX_W1) & _M32
    return c0, c1, c2, c3


def class_scores(N: int, seed: int, step: int) -> np.ndarray:
    """32-bit random score of every class id 0..N-1 for one iteration.

    Class j takes word (j mod 4) of the Philox block whose counter is
    (lo32(j div 4), hi32(j div 4), lo32(step), hi32(step)) under key (lo32(seed), hi32(seed)).
    The iteration number is part of the counter because the paper re-draws the negatives
    "in every iteration" (Sec. 3.2).
    """
    nq = (N + 3) // 4
    q = np.arange(nq, dtype=np.uint64)
    step = int(step) & 0xFFFFFFFFFFFFFFFF
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    words = philox4x32_10(
        (q & _M32, q >> _S32, np.uint64(step & 0xFFFFFFFF), np.uint64(step >> 32)),
        (np.uint64(seed & 0xFFFFFFFF), np.uint64(seed >> 32)),
    )
    u = np.stack([np.broadcast_to(w, q.shape) for w in words], axis=1).reshape(-1)
    return u[:N].astype(np.uint32)


def num_sampled(N: int, r: float, U: int) -> int:
    """|S| = C*r (text after Eq. 4), never fewer than the U classes present in the batch
    (Sec. 3.3: the minimum ratio keeps just the within-batch classes)."""
    return max(int(U), int(math.ceil(float(r) * float(N))))


def sample(labels, N: int, r: float, seed: int, step: int, score_mask: int = 0xFFFFFFFF):
    """Sampled class set S of one iteration (Sec. 3.2, Fig. 4).

    Returns (idx int32[k] ascending, y_local int32[B], k).  Total order on classes:
    positives first, then larger score, then smaller class id; S is its first k elements.
    `score_mask` is ANDed onto every score (test hook to force ties; all ones normally).
    """
    labels = np.asarray(labels, dtype=np.int64)
    if labels.ndim != 1 or labels.size < 1:
        raise ValueError("labels must be a non-empty vector")
    if labels.min() < 0 or labels.max() >= N:
        raise ValueError("label outside [0, N)")
    if not (0.0 < r <= 1.0):
        raise ValueError("r must be in (0, 1]")
    pos = np.zeros(N, dtype=bool)
    pos[labels] = True
    U = int(pos.sum())
    k = num_sampled(N, r, U)
    u = class_scores(N, seed, step) & np.uint32(score_mask)
    j = np.arange(N, dtype=np.int64)
    # np.lexsort: the LAST key is the primary one.  Ascending on (not pos, -score, id).
    order = np.lexsort((j, -u.astype(np.int64), ~pos))
    idx = np.sort(order[:k]).astype(np.int32)
    y_local = np.searchsorted(idx, labels).astype(np.int32)
    return idx, y_local, k


def forward_backward(X, W_S, y_local, s: float, m: float, margin: str = "arcface",
                     filter_threshold=None):
    """Margin-softmax loss over the sampled centers and all its gradients, in fp64.

    X: B x D raw features; W_S: k x D raw sampled centers (rows W[idx]); y_local[i] is the
    row of W_S that is sample i's own class.  Follows Eq. 1 (loss, mean over B) with the
    label logit replaced by the margin-based one, and Eq. 2-4 by the chain rule.

    margin: "arcface"  label logit s*cos(theta + m)  (additive angular margin), or
            "cosface"  label logit s*(cos(theta) - m) (additive cosine margin);
            Sec. 4.1 trains with the hyper-parameters of both papers.
    filter_threshold: the PFC* variant of Sec. 3.3 / Fig. 4 caption: a NEGATIVE center whose
            cosine to the sample exceeds the fixed threshold (0.4 in the paper) is left out of that
            sample's softmax.  None keeps every center.  The mask is a function of the clamped cosine; it is constant in a
            neighbourhood of almost every input, so it carries no gradient of its own.

    Returns a dict:
      loss                      scalar
      cos (B x k, clamped), z (B x k logits; -inf where filtered), lse (B), p (B x k)
      dc  (B x k)               dL/d cos
      dXn (B x D), dWn (k x D)  gradients w.r.t. the normalised rows
      u (B), t (k)              dXn_i . xn_i  and  dWn_j . wn_j
      dX (B x D), dW (k x D)    gradients w.r.t. the raw rows
      xn, wn, x_norm, w_norm
      apcs                      mean over the batch of the label cosine        (Sec. 3.3)
      amncs                     mean over the batch of the largest cosine to a sampled center
                                other than the label's, taken before any filtering (Sec. 3.3)
    """
    X = np.asarray(X, dtype=np.float64)
    W_S = np.asarray(W_S, dtype=np.float64)
    y = np.asarray(y_local, dtype=np.int64)
    B, D = X.shape
    k = W_S.shape[0]
    if W_S.shape[1] != D or y.shape != (B,):
        raise ValueError("shape mismatch")
    if y.min() < 0 or y.max() >= k:
        raise ValueError("y_local outside [0, k)")
    if margin not in ("arcface", "cosface"):
        raise ValueError("unknown margin")
    rows = np.arange(B)

    x_norm = np.maximum(np.sqrt((X * X).sum(axis=1)), EPS_NORM)
    w_norm = np.maximum(np.sqrt((W_S * W_S).sum(axis=1)), EPS_NORM)
    xn = X / x_norm[:, None]
    wn = W_S / w_norm[:, None]

    c = np.clip(xn @ wn.T, -1.0, 1.0)
    onehot = np.zeros((B, k), dtype=bool)
    onehot[rows, y] = True
    z = s * c
    c_lab = c[rows, y]
    if margin == "arcface":
        sin_lab = np.sqrt(1.0 - c_lab * c_lab)
        z[rows, y] = s * (c_lab * math.cos(m) - sin_lab * math.sin(m))   # s*cos(theta+m)
        # d cos(theta+m) / d cos(theta) = sin(theta+m)/sin(theta)
        rho = math.cos(m) + c_lab * math.sin(m) / np.sqrt(np.maximum(1.0 - c_lab * c_lab, EPS_SIN2))
    else:
        z[rows, y] = s * (c_lab - m)
        rho = np.ones(B)
    keep = np.ones((B, k), dtype=bool)
    if filter_threshold is not None:
        keep = onehot | ~(c > float(filter_threshold))
        z = np.where(keep, z, -np.inf)

    zmax = z.max(axis=1)
    lse = zmax + np.log(np.exp(z - zmax[:, None]).sum(axis=1))
    loss = float((lse - z[rows, y]).sum() / B)

    p = np.exp(z - lse[:, None])       # exactly 0 where filtered
    dz = p.copy()
    dz[rows, y] -= 1.0
    dz /= B
    dc = s * dz
    dc[rows, y] *= rho

    dXn = dc @ wn
    dWn = dc.T @ xn
    u = (dXn * xn).sum(axis=1)
    t = (dWn * wn).sum(axis=1)
    dX = (dXn - u[:, None] * xn) / x_norm[:, None]
    dW = (dWn - t[:, None] * wn) / w_norm[:, None]

    apcs = float(c_lab.mean())
    if k > 1:
        amncs = float(np.where(onehot, -np.inf, c).max(axis=1).mean())
    else:
        amncs = float("nan")
    return dict(loss=loss, cos=c, z=z, lse=lse, p=p, dc=dc, dXn=dXn, dWn=dWn, u=u, t=t,
                dX=dX, dW=dW, xn=xn, wn=wn, x_norm=x_norm, w_norm=w_norm, apcs=apcs, amncs=amncs,
                keep=keep)


def update(W, v, idx, dW, lr: float, mu: float) -> None:
    """SGD-with-momentum step on the sampled rows only, in place (Eq. 3 with a momentum
    buffer; text after Eq. 4: only the sampled centers are updated).  W, v: N x D (or any
    array indexable by idx); rows outside idx are not read or written."""
    idx = np.asarray(idx, dtype=np.int64)
    v_new = mu * v[idx] + dW
    v[idx] = v_new
    W[idx] = W[idx] - lr * v_new


def step(X, labels, W, v, *, r, s, m, lr, mu, seed, step):
    """One whole PFC iteration on full N x D arrays W, v (updated in place).
    Returns (loss, dX, idx, y_local, fb) where fb is forward_backward's dict."""
    N = W.shape[0]
    idx, y_local, _k = sample(labels, N, r, seed, step)
    fb = forward_backward(X, W[idx.astype(np.int64)], y_local, s, m)
    update(W, v, idx, fb["dW"], lr, mu)
    return fb["loss"], fb["dX"], idx, y_local, fb
