"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI and the oracle on
the same seeded inputs.  Nothing here computes any part of the method."""
from __future__ import annotations

import numpy as np

from paper_2203_15565_amd import binding


def torch_mod():
    import torch
    return torch


def gpu_sample(ctx, labels_np, r, seed, step, score_mask=None):
    """Returns (idx int32[k], y_local int32[B], k) as NumPy arrays from pfc_sample."""
    torch = torch_mod()
    B = labels_np.size
    cap = binding.pfc_num_sampled(ctx.N, B, r)
    labels = torch.from_numpy(np.ascontiguousarray(labels_np, dtype=np.int64)).cuda()
    idx = torch.full((cap,), -7, dtype=torch.int32, device="cuda")
    yl = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    k = ctx.pfc_sample(labels, r, seed, step, idx, yl, score_mask=score_mask)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), yl.cpu().numpy(), k


def gpu_forward_backward(ctx, X_np, W_dev, idx_np, yl_np, s, m):
    """W_dev: torch fp32 [N x D] on the GPU.  Returns (loss, dX, dWn) as NumPy."""
    torch = torch_mod()
    B, D = X_np.shape
    k = idx_np.size
    X = torch.from_numpy(np.ascontiguousarray(X_np, dtype=np.float32)).cuda()
    idx = torch.from_numpy(np.ascontiguousarray(idx_np, dtype=np.int32)).cuda()
    yl = torch.from_numpy(np.ascontiguousarray(yl_np, dtype=np.int32)).cuda()
    loss = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    dX = torch.full((B, D), float("nan"), dtype=torch.float32, device="cuda")
    dW = torch.full((k, D), float("nan"), dtype=torch.float32, device="cuda")
    ctx.pfc_forward_backward(X, W_dev, idx, k, yl, s, m, loss, dX, dW)
    torch.cuda.synchronize()
    return float(loss.item()), dX.cpu().numpy(), dW.cpu().numpy()


def rel_max(a, b):
    """max |a-b| / max |b|"""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-300))


def row_rel_err(W_gpu, W_ref, ref_norm):
    """max over rows of max|row diff| / |reference row|  (the bar for updated centers)."""
    d = np.abs(np.asarray(W_gpu, dtype=np.float64) - np.asarray(W_ref, dtype=np.float64)).max(axis=1)
    return float((d / ref_norm).max())


# Per-row gradient bars.  A center that is nobody's label has a gradient row whose largest entry
# is only a few percent of the largest entry of the whole matrix (the label rows dominate), so a
# bar relative to the global maximum says little about it; these bars are relative to each row's
# own largest entry.  What sets them is the logit, not the sum over the batch: such a row is
# often dominated by ONE sample, dWn_j ~ (s/B) p_ij xn_i, and p_ij = exp(s cos_ij)/l_i carries the
# error of the cosine multiplied by s.  With bf16 operands every product xn_d wn_d is off by about
# 2^-9 sqrt(2/3) relative, the sum over D = 512 terms of size 1/D by 7e-5, hence s |d cos| = 4.5e-3
# rms at s = 64; the worst of the 4e7 .. 1e9 (sample, center) pairs of the workloads lies 5.5 to 6
# standard deviations out: 2.5e-2 .. 3e-2 observed, bar 5e-2.  fp32 operands: s * 1e-7, bar 1e-4.
# Rows whose largest oracle entry is below ROW_FLOOR of the matrix's largest entry are left to the
# global bar (nothing relative can be said about a row of zeros).
ROW_GRAD_TOL = {binding.PRECISION_FP32: 1e-4, binding.PRECISION_BF16: 5e-2}
ROW_FLOOR = 1e-6


def dim_amp(precision, D):
    """Factor on the bf16 gradient bars for rows shorter than the D = 512 they were derived at:
    the rounding error of a cosine is that of a sum of D products of size 1/D, i.e. it grows as
    1/sqrt(D) when D shrinks (3.6e-4 at D = 64 against 1.3e-4 rms at D = 512 in units of the
    cosine).  Longer rows keep the D = 512 bars; fp32 operands are not affected at these bars."""
    if precision != binding.PRECISION_BF16 or D >= 512:
        return 1.0
    return float(np.sqrt(512.0 / D))


def row_rel_max(a, b, floor=ROW_FLOOR):
    """max over rows of max|a_row - b_row| / max|b_row|, rows of b below floor * max|b| excluded.
    Returns (worst ratio, number of rows compared)."""
    a = np.asarray(a)
    b = np.asarray(b)
    worst, count = 0.0, 0
    gmax = float(np.abs(b).max())
    step = max(1, (1 << 24) // max(1, b.shape[1]))       # bounded fp64 temporaries
    for r0 in range(0, b.shape[0], step):
        bb = b[r0:r0 + step].astype(np.float64)
        d = np.abs(a[r0:r0 + step].astype(np.float64) - bb).max(axis=1)
        rmax = np.abs(bb).max(axis=1)
        ok = rmax >= floor * gmax
        if ok.any():
            worst = max(worst, float((d[ok] / rmax[ok]).max()))
            count += int(ok.sum())
    return worst, count
