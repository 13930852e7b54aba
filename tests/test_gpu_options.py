"""GPU parity of pfc_forward_backward_ex: CosFace margin, the PFC* filter and APCS / AMNCS
(arXiv 2203.15565, Sec. 4.1; Sec. 3.3 and Fig. 4 caption)."""
import math
import sys

import numpy as np
import pytest

from oracle import pfc_oracle as O
from paper_2203_15565_amd import binding
from pfc_harness import gpu_sample, rel_max

pytestmark = pytest.mark.gpu

LOSS_TOL = {binding.PRECISION_FP32: 1e-5, binding.PRECISION_BF16: 2e-3}
GRAD_TOL = {binding.PRECISION_FP32: 2e-5, binding.PRECISION_BF16: 1e-2}


def _say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _run_ex(precision, N, B, D, r, s, m, margin, thr, seed, wscale=0.01, clusters=0, want_stats=True):
    import torch
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((N, D)) * wscale).astype(np.float32)
    labels = rng.integers(0, N, size=B)
    X = rng.standard_normal((B, D)).astype(np.float32)
    if clusters:
        # features close to a few class centers: several cosines well above the 0.4 threshold
        pick = rng.integers(0, N, size=B)
        X = (W[pick] / np.linalg.norm(W[pick], axis=1, keepdims=True) * 3.0 +
             rng.standard_normal((B, D)).astype(np.float32) * (3.0 / math.sqrt(D))).astype(np.float32)
        labels[: B // 2] = pick[: B // 2]
    ctx = binding.Context(N, D, B, r, precision)
    idx, yl, k = gpu_sample(ctx, labels, r, 0, 0)
    idx = idx[:k]
    Xd, Wd = torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda()
    idx_d, yl_d = torch.from_numpy(idx).cuda(), torch.from_numpy(yl).cuda()
    loss = torch.zeros(1, device="cuda")
    dX = torch.zeros(B, D, device="cuda")
    dW = torch.zeros(k, D, device="cuda")
    stats = torch.full((2,), float("nan"), device="cuda") if want_stats else None
    mt = binding.MARGIN_COSFACE if margin == "cosface" else binding.MARGIN_ARCFACE
    _say("options", precision, N, B, D, margin, thr, "k", k)
    ctx.pfc_forward_backward_ex(Xd, Wd, idx_d, k, yl_d, s, m, mt, 2.0 if thr is None else thr, loss,
                                dX, dW, stats)
    torch.cuda.synchronize()
    assert ctx.pfc_check() == binding.PFC_OK
    o = O.forward_backward(X, W[idx.astype(np.int64)], yl, s, m, margin=margin, filter_threshold=thr)
    if thr is not None:
        # the filter decides on the cosine: pairs within rounding distance of the threshold may
        # legitimately fall on either side, so the case must not contain any
        gap = {binding.PRECISION_FP32: 1e-5, binding.PRECISION_BF16: 4e-3}[precision]
        assert np.abs(o["cos"] - thr).min() > gap, "test case has a cosine on the threshold"
    gl = float(loss.item())
    _say("   loss", gl, o["loss"], "filtered pairs", int((~o["keep"]).sum()))
    assert abs(gl - o["loss"]) <= LOSS_TOL[precision] * abs(o["loss"])
    amp = max(1.0, s / 64.0)       # the error of a logit is s * (error of the cosine)
    assert rel_max(dX.cpu().numpy(), o["dX"]) <= GRAD_TOL[precision] * amp
    assert rel_max(dW.cpu().numpy(), o["dWn"]) <= GRAD_TOL[precision] * amp
    if want_stats:
        st = stats.cpu().numpy()
        tol = 1e-5 if precision == binding.PRECISION_FP32 else 2e-3
        assert abs(st[0] - o["apcs"]) <= tol and abs(st[1] - o["amncs"]) <= tol, (st, o["apcs"], o["amncs"])
    ctx.close()
    return o


@pytest.mark.parametrize("precision", [binding.PRECISION_FP32, binding.PRECISION_BF16])
def test_cosface(precision):
    _run_ex(precision, 6000, 96, 512, 0.1, 64.0, 0.4, "cosface", None, seed=31)
    _run_ex(precision, 3000, 70, 256, 0.2, 30.0, 0.35, "cosface", None, seed=32, wscale=1.0)


@pytest.mark.parametrize("precision", [binding.PRECISION_FP32, binding.PRECISION_BF16])
def test_pfc_star_filter(precision):
    o = _run_ex(precision, 2000, 128, 256, 0.25, 32.0, 0.5, "arcface", 0.4, seed=33, clusters=1)
    assert (~o["keep"]).sum() > 10            # the filter really removed pairs
    o = _run_ex(precision, 2000, 128, 256, 0.25, 32.0, 0.4, "cosface", 0.4, seed=34, clusters=1)
    assert (~o["keep"]).sum() > 10


@pytest.mark.parametrize("precision", [binding.PRECISION_FP32, binding.PRECISION_BF16])
def test_filter_at_a_scale_above_64(precision):
    """The per-sample reference of the softmax (scales above 64) must be the largest logit among
    the entries the filter KEEPS: here the largest cosines of many samples are filtered ones."""
    o = _run_ex(precision, 2000, 128, 256, 0.25, 160.0, 0.5, "arcface", 0.4, seed=36, clusters=1)
    assert (~o["keep"]).sum() > 10
    kept_max = np.where(o["keep"], o["z"], -np.inf).max(axis=1)
    all_max = (160.0 * o["cos"]).max(axis=1)
    assert (all_max - kept_max > 88.0).any()      # a reference over all entries would underflow


@pytest.mark.parametrize("precision", [binding.PRECISION_FP32, binding.PRECISION_BF16])
def test_filter_off_equals_plain_call(precision):
    """threshold >= 1 and no stats: bit-identical to pfc_forward_backward."""
    import torch
    N, B, D, r = 5000, 64, 512, 0.1
    rng = np.random.default_rng(35)
    X = rng.standard_normal((B, D)).astype(np.float32)
    W = (rng.standard_normal((N, D)) * 0.01).astype(np.float32)
    labels = rng.integers(0, N, size=B)
    ctx = binding.Context(N, D, B, r, precision)
    idx, yl, k = gpu_sample(ctx, labels, r, 0, 0)
    Xd, Wd = torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda()
    idx_d, yl_d = torch.from_numpy(idx[:k]).cuda(), torch.from_numpy(yl).cuda()
    outs = []
    for call in range(3):
        loss = torch.zeros(1, device="cuda")
        dX = torch.zeros(B, D, device="cuda")
        dW = torch.zeros(k, D, device="cuda")
        if call == 0:
            ctx.pfc_forward_backward(Xd, Wd, idx_d, k, yl_d, 64.0, 0.5, loss, dX, dW)
        elif call == 1:
            ctx.pfc_forward_backward_ex(Xd, Wd, idx_d, k, yl_d, 64.0, 0.5, binding.MARGIN_ARCFACE, 1.0,
                                        loss, dX, dW, None)
        else:   # stats requested: the extras path, same numbers
            st = torch.zeros(2, device="cuda")
            ctx.pfc_forward_backward_ex(Xd, Wd, idx_d, k, yl_d, 64.0, 0.5, binding.MARGIN_ARCFACE, 1.5,
                                        loss, dX, dW, st)
        torch.cuda.synchronize()
        outs.append((loss.cpu().numpy().tobytes(), dX.cpu().numpy().tobytes(), dW.cpu().numpy().tobytes()))
    assert outs[0] == outs[1] == outs[2]
    ctx.close()


def test_ex_einval():
    import torch
    ctx = binding.Context(1000, 512, 8, 0.1, binding.PRECISION_FP32)
    X = torch.zeros(8, 512, device="cuda")
    W = torch.zeros(1000, 512, device="cuda")
    idx = torch.arange(100, dtype=torch.int32, device="cuda")
    yl = torch.zeros(8, dtype=torch.int32, device="cuda")
    loss = torch.zeros(1, device="cuda")
    dX = torch.zeros(8, 512, device="cuda")
    dW = torch.zeros(100, 512, device="cuda")
    for mt, thr in ((2, 0.4), (-1, 0.4), (0, float("nan")), (0, -1.5)):
        with pytest.raises(binding.PfcError) as e:
            ctx.pfc_forward_backward_ex(X, W, idx, 100, yl, 64.0, 0.5, mt, thr, loss, dX, dW, None)
        assert e.value.code == binding.PFC_EINVAL
    ctx.close()
