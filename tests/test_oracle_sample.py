"""Pins of the oracle's sampler (CPU only).

Cited passages are of arXiv 2203.15565: Sec. 3.2 (positives first, random negatives fill
the buffer, |S| = C*r), Sec. 3.3 (minimum ratio keeps only within-batch classes), text after
Eq. 4 (update frequency of a center falls from 1 to r).
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import pfc_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _scalar_philox(counter, key):
    """Independent scalar restatement with Python integers (no NumPy), used as brute force."""
    c = list(counter)
    k = list(key)
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & 0xFFFFFFFF, p1 & 0xFFFFFFFF,
             ((p0 >> 32) ^ c[3] ^ k[1]) & 0xFFFFFFFF, p0 & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def test_philox_known_answers():
    n = 0
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            lhs, rhs = line.split("->")
            w = [int(t, 16) for t in lhs.split()]
            exp = [int(t, 16) for t in rhs.split()]
            got = [int(x) for x in O.philox4x32_10(w[:4], w[4:])]
            assert got == exp
            assert _scalar_philox(w[:4], w[4:]) == exp
            n += 1
    assert n == 3


def test_philox_vectorised_matches_scalar():
    rng = np.random.default_rng(7)
    ctr = rng.integers(0, 2**32, size=(4, 50), dtype=np.uint64)
    key = rng.integers(0, 2**32, size=2, dtype=np.uint64)
    out = O.philox4x32_10(tuple(ctr), tuple(key))
    for i in range(50):
        exp = _scalar_philox([int(ctr[j, i]) for j in range(4)], [int(key[0]), int(key[1])])
        assert [int(out[j][i]) for j in range(4)] == exp


def test_class_scores_layout():
    """Class j takes word j%4 of the block with counter (j//4, 0, lo(step), hi(step))."""
    seed = 0x1234567890ABCDEF
    step = (5 << 32) | 9
    N = 23
    u = O.class_scores(N, seed, step)
    assert u.dtype == np.uint32 and u.shape == (N,)
    for j in range(N):
        blk = _scalar_philox([j // 4, 0, 9, 5], [seed & 0xFFFFFFFF, seed >> 32])
        assert int(u[j]) == blk[j % 4]
    # a different iteration or seed gives different scores
    assert (O.class_scores(N, seed, step + 1) != u).any()
    assert (O.class_scores(N, seed + 1, step) != u).any()


def test_num_sampled_golden():
    with open(os.path.join(GOLDEN, "num_sampled.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            N, p, q, exp = [int(t) for t in line.split()]
            exact = math.ceil(Fraction(N * p, q))
            assert exact == exp
            assert O.num_sampled(N, p / q, 0) == exp
            assert O.num_sampled(N, p / q, exp + 5) == exp + 5   # never fewer than U


def _brute_sample(labels, N, r, seed, step, mask=0xFFFFFFFF):
    pos = set(int(l) for l in labels)
    k = max(len(pos), math.ceil(r * N))
    keyed = []
    for j in range(N):
        blk = _scalar_philox([j // 4, 0, step & 0xFFFFFFFF, step >> 32],
                             [seed & 0xFFFFFFFF, seed >> 32])
        u = blk[j % 4] & mask
        keyed.append((0 if j in pos else 1, -u, j))
    chosen = sorted(t[2] for t in sorted(keyed)[:k])
    return chosen, [chosen.index(int(l)) for l in labels]


@pytest.mark.parametrize("N,B,r", [(64, 4, 0.25), (61, 7, 0.1), (17, 5, 0.5), (40, 3, 1.0),
                                   (33, 9, 0.05)])
def test_sample_matches_brute_force(N, B, r):
    rng = np.random.default_rng(N * 1000 + B)
    for step in range(3):
        labels = rng.integers(0, N, size=B)
        idx, yl, k = O.sample(labels, N, r, seed=11, step=step)
        bidx, byl = _brute_sample(labels, N, r, 11, step)
        assert idx.tolist() == bidx
        assert yl.tolist() == byl
        assert k == len(bidx)


def test_sample_invariants():
    N, B, r = 5000, 64, 0.1
    rng = np.random.default_rng(3)
    labels = rng.integers(0, N, size=B)
    labels[:8] = labels[8]          # duplicates
    idx, yl, k = O.sample(labels, N, r, seed=0, step=0)
    U = len(set(labels.tolist()))
    assert k == max(U, math.ceil(r * N)) == idx.size
    assert idx.dtype == np.int32 and yl.dtype == np.int32
    assert (np.diff(idx) > 0).all() and idx[0] >= 0 and idx[-1] < N
    assert set(labels.tolist()) <= set(idx.tolist())
    assert (idx[yl] == labels).all()
    # deterministic in (seed, step); negatives change with the iteration
    idx2, _, _ = O.sample(labels, N, r, seed=0, step=0)
    assert (idx == idx2).all()
    idx3, _, _ = O.sample(labels, N, r, seed=0, step=1)
    assert set(idx3.tolist()) != set(idx.tolist())
    assert set(labels.tolist()) <= set(idx3.tolist())


def test_sample_negatives_are_top_scores():
    """Every chosen negative scores at least as high as every rejected class."""
    N, B, r = 3000, 32, 0.2
    labels = np.random.default_rng(5).integers(0, N, size=B)
    idx, _, _ = O.sample(labels, N, r, seed=9, step=4)
    u = O.class_scores(N, 9, 4).astype(np.int64)
    chosen = np.zeros(N, bool)
    chosen[idx] = True
    pos = np.zeros(N, bool)
    pos[labels] = True
    neg_in = chosen & ~pos
    out = ~chosen
    assert u[neg_in].min() >= u[out].max()


def test_sample_r_one_is_every_class():
    N = 257
    labels = np.array([3, 3, 200, 256])
    idx, yl, k = O.sample(labels, N, 1.0, seed=1, step=0)
    assert k == N and (idx == np.arange(N)).all() and (yl == labels).all()


def test_sample_minimum_ratio_keeps_only_batch_classes():
    """Sec. 3.3: at the minimum ratio no negative outside the batch is drawn."""
    N = 1000
    labels = np.array([5, 900, 5, 17, 333, 17, 999, 0])
    idx, yl, k = O.sample(labels, N, 0.001, seed=2, step=7)     # ceil(rN) = 1 < U = 6
    assert idx.tolist() == sorted(set(labels.tolist()))
    assert k == 6 and (idx[yl] == labels).all()


def test_sample_forced_ties_take_lowest_ids():
    N = 100
    labels = np.array([90, 95])
    idx, _, k = O.sample(labels, N, 0.1, seed=0, step=0, score_mask=0)
    assert k == 10
    assert idx.tolist() == list(range(8)) + [90, 95]
    # partial ties: keep only the top 2 bits of each score -> many equal keys
    idx2, _, _ = O.sample(labels, N, 0.3, seed=0, step=0, score_mask=0xC0000000)
    bidx, _ = _brute_sample(labels, N, 0.3, 0, 0, mask=0xC0000000)
    assert idx2.tolist() == bidx


def test_sample_negative_inclusion_frequency():
    """Text after Eq. 4: a center is touched with frequency r; for a never-positive class the
    inclusion probability is (k - U)/(N - U)."""
    N, r, steps = 400, 0.25, 4000
    labels = np.array([1, 2, 3, 4])
    k = math.ceil(r * N)
    count = np.zeros(N)
    for t in range(steps):
        idx, _, _ = O.sample(labels, N, r, seed=123, step=t)
        count[idx] += 1
    freq = count / steps
    assert (freq[labels] == 1.0).all()
    neg = np.ones(N, bool)
    neg[labels] = False
    pexp = (k - 4) / (N - 4)
    sigma = math.sqrt(pexp * (1 - pexp) / steps)
    assert abs(freq[neg].mean() - pexp) < 1e-12          # exactly k-U negatives each step
    assert np.abs(freq[neg] - pexp).max() < 5.5 * sigma  # per-class frequencies


def test_sample_rejects_bad_input():
    with pytest.raises(ValueError):
        O.sample(np.array([0, 10]), 10, 0.5, 0, 0)
    with pytest.raises(ValueError):
        O.sample(np.array([0, -1]), 10, 0.5, 0, 0)
    with pytest.raises(ValueError):
        O.sample(np.array([0]), 10, 0.0, 0, 0)
    with pytest.raises(ValueError):
        O.sample(np.array([0]), 10, 1.5, 0, 0)
