"""CPU checks of the comparison helpers the GPU parity tests rely on: the row-by-row gradient bar
must catch a mistake in the gradient of a center that is nobody's label, which the bar relative to
the largest entry of the whole matrix lets through.  The mistake is planted in a copy of the
oracle's own result; no kernel is involved."""
import numpy as np

from oracle import pfc_oracle as O
from paper_2203_15565_amd import binding
from pfc_harness import ROW_GRAD_TOL, rel_max, row_rel_max

GLOBAL_BF16_TOL = 1e-2     # the bar against the largest entry of the matrix (tests/test_gpu_step.py)


def _oracle_case(N=10_000, B=128, D=512, r=0.1, seed=5):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((B, D))
    W = rng.standard_normal((N, D)) * 0.01
    labels = rng.integers(0, N, size=B)
    idx, yl, k = O.sample(labels, N, r, 0, 0)
    return O.forward_backward(X, W[idx.astype(np.int64)], yl, 64.0, 0.5), yl, k


def test_negative_rows_are_small_against_the_largest_entry():
    """Why a per-row bar is needed at all: the typical row of a never-positive center peaks at a
    few percent of the matrix's largest entry (which sits in a label row)."""
    o, yl, k = _oracle_case()
    g = np.abs(o["dWn"])
    neg = np.setdiff1d(np.arange(k), yl)
    ratio = np.median(g[neg].max(axis=1)) / g.max()
    assert 0.002 < ratio < 0.1, ratio


def test_wrong_negative_row_fails_the_row_bar_but_passes_the_global_one():
    o, yl, k = _oracle_case()
    ref = o["dWn"]
    neg = np.setdiff1d(np.arange(k), yl)
    j = neg[np.argsort(np.abs(ref[neg]).max(axis=1))[neg.size // 2]]     # the median negative row
    bad = ref.copy()
    bad[j] *= 1.1                                     # that center's gradient is 10 % too long
    assert rel_max(bad, ref) <= GLOBAL_BF16_TOL       # invisible against the largest entry
    worst, n = row_rel_max(bad, ref)
    assert n == k
    assert worst > ROW_GRAD_TOL[binding.PRECISION_BF16]        # caught row by row
    assert abs(worst - 0.1) < 1e-9
    # a dropped sample in one negative row (one term of the sum over the batch missing)
    bad = ref.copy()
    i = int(np.argsort(o["dc"][:, j])[-4])            # one of the larger terms, not the largest
    bad[j] -= o["dc"][i, j] * o["xn"][i]
    assert rel_max(bad, ref) <= GLOBAL_BF16_TOL
    assert row_rel_max(bad, ref)[0] > ROW_GRAD_TOL[binding.PRECISION_BF16]


def test_row_bar_accepts_rounding_sized_noise_and_skips_empty_rows():
    o, yl, k = _oracle_case()
    ref = o["dWn"]
    rng = np.random.default_rng(1)
    # bf16-sized relative noise on every entry stays inside the bf16 row bar
    noisy = ref * (1.0 + rng.uniform(-1, 1, ref.shape) * 2.0 ** -8)
    assert row_rel_max(noisy, ref)[0] <= ROW_GRAD_TOL[binding.PRECISION_BF16]
    # an all-zero reference row is left to the global bar, not divided by
    ref2 = ref.copy()
    ref2[3] = 0.0
    worst, n = row_rel_max(ref2, ref2)
    assert worst == 0.0 and n == k - 1
    assert row_rel_max(ref.astype(np.float32), ref)[0] <= ROW_GRAD_TOL[binding.PRECISION_FP32]
