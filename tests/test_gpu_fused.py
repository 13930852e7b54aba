"""GPU parity of pfc_forward_backward_update (forward/backward and update in one call): against
the oracle, and against the two separate calls it stands for."""
from __future__ import annotations

import sys

import numpy as np
import pytest

from oracle import pfc_oracle as O
from paper_2203_15565_amd import binding, workloads
from pfc_harness import ROW_GRAD_TOL, rel_max, row_rel_err, row_rel_max
from test_gpu_step import (FULL_SIZE, GRAD_TOL, LOSS_TOL, W_TOL, _device_weight, _run_steps,
                           _weight_cache)

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, file=sys.stderr, flush=True)


def _torch():
    import torch
    return torch


# (N, B, D, r, precision, label spread).  D = 512 with at least one 128-row tile per compute unit
# (k >= 32K on a 256-CU GPU) takes the one-kernel form, the rows beyond the last whole round of
# tiles going to half-height tiles; everything else goes through the context's gradient buffer.
CASES = [
    (400_000, 300, 512, 0.1, binding.PRECISION_BF16, 400_000),  # one kernel, ragged B, k and tail
    (400_000, 300, 512, 0.1, binding.PRECISION_FP32, 60),       # one kernel, heavy duplicates
    (327_680, 256, 512, 0.1, binding.PRECISION_BF16, 327_680),  # one kernel, k = 32768: no tail
    (1_000_003, 300, 512, 0.1, binding.PRECISION_BF16, 1_000_003),  # one kernel, three rounds of tiles
    (10_000, 128, 512, 0.1, binding.PRECISION_FP32, 10_000),    # too few tiles
    (93_431, 512, 512, 0.1, binding.PRECISION_BF16, 93_431),
    (3_000, 100, 256, 0.1, binding.PRECISION_FP32, 3_000),      # D != 512
    (5_000, 70, 1024, 0.2, binding.PRECISION_BF16, 5_000),      # D = 1024
    (4_000, 33, 768, 0.15, binding.PRECISION_FP32, 40),         # D = 768, duplicates
    (50_000, 4096, 512, 1e-9, binding.PRECISION_BF16, 50_000),  # k = U small, batch sliced
    (50_000, 3000, 512, 1e-9, binding.PRECISION_FP32, 40),      # three label windows, 40 classes
    (400_000, 2100, 512, 0.1, binding.PRECISION_BF16, 300),     # one kernel, three label windows
    (6_000, 100, 192, 0.1, binding.PRECISION_BF16, 6_000),      # D a multiple of 64 only
    (50_000, 4096, 128, 1e-9, binding.PRECISION_FP32, 50_000),  # likewise, batch sliced
]


@pytest.mark.parametrize("N,B,D,r,precision,spread", CASES)
@pytest.mark.parametrize("options", [False, True])
def test_fused_equals_two_calls(N, B, D, r, precision, spread, options):
    torch = _torch()
    rng = np.random.default_rng(77)
    W0 = (rng.standard_normal((N, D)) * 0.01).astype(np.float32)
    v0 = (rng.standard_normal((N, D)) * 1e-3).astype(np.float32)
    X = rng.standard_normal((B, D)).astype(np.float32)
    labels = rng.permutation(N)[:spread][rng.integers(0, spread, size=B)].astype(np.int64)
    s, m, lr, mu = 64.0, 0.5, 0.1, 0.9
    margin = binding.MARGIN_COSFACE if options else binding.MARGIN_ARCFACE
    tau = 0.05 if options else 2.0
    if options:
        m = 0.35
    out = {}
    for fused in (False, True):
        _say("fused vs two calls", N, B, D, r, precision, spread, options, "fused" if fused else "split")
        ctx = binding.Context(N, D, B, r, precision)
        Wd, vd = torch.from_numpy(W0).cuda(), torch.from_numpy(v0).cuda()
        cap = binding.pfc_num_sampled(N, B, r)
        idx = torch.zeros(cap, dtype=torch.int32, device="cuda")
        yl = torch.zeros(B, dtype=torch.int32, device="cuda")
        loss = torch.zeros(1, device="cuda")
        dX = torch.zeros(B, D, device="cuda")
        stats = torch.zeros(2, device="cuda") if options else None
        Xd, ld = torch.from_numpy(X).cuda(), torch.from_numpy(labels).cuda()
        k = ctx.pfc_sample(ld, r, 3, 5, idx, yl)
        if fused:
            ctx.pfc_forward_backward_update(Xd, Wd, vd, idx, k, yl, s, m, lr, mu, loss, dX,
                                            margin_type=margin, filter_threshold=tau,
                                            stats_out=stats)
        else:
            dW = torch.zeros(cap, D, device="cuda")
            ctx.pfc_forward_backward_ex(Xd, Wd, idx, k, yl, s, m, margin, tau, loss, dX, dW, stats)
            ctx.pfc_update(Wd, vd, idx, k, dW, lr, mu)
        torch.cuda.synchronize()
        assert ctx.pfc_check() == binding.PFC_OK
        out[fused] = (Wd.cpu().numpy(), vd.cpu().numpy(), float(loss.item()), dX.cpu().numpy(),
                      None if stats is None else stats.cpu().numpy(), idx[:k].cpu().numpy())
        ctx.close()
    Wa, va, la, dXa, sa, ia = out[False]
    Wb, vb, lb, dXb, sb, ib = out[True]
    assert np.array_equal(ia, ib)
    # loss, feature gradient and statistics come from the same kernels on the same inputs
    assert la == lb
    assert dXa.tobytes() == dXb.tobytes()
    if options:
        assert sa.tobytes() == sb.tobytes()
    # rows outside the sample: untouched by both
    mask = np.ones(N, dtype=bool)
    mask[ia] = False
    assert Wb[mask].tobytes() == W0[mask].tobytes() and vb[mask].tobytes() == v0[mask].tobytes()
    # sampled rows: same arithmetic up to the summation order inside the GEMM tiles
    sel = ia.astype(np.int64)
    assert not np.array_equal(Wb[sel], W0[sel])
    nrm = np.linalg.norm(Wa[sel].astype(np.float64), axis=1)
    err = row_rel_err(Wb[sel], Wa[sel], nrm)
    _say("   W row diff fused vs two calls", err, "identical" if Wa.tobytes() == Wb.tobytes() else "")
    assert err <= 1e-6
    assert rel_max(vb[sel], va[sel]) <= 1e-5
    # row by row: the two forms differ only in the summation order inside the GEMM tiles
    rv, nv = row_rel_max(vb[sel], va[sel])
    _say("   v per-row diff fused vs two calls", rv)
    assert rv <= 1e-4 and nv >= 0.9 * sel.size


@pytest.mark.parametrize("precision", [binding.PRECISION_FP32, binding.PRECISION_BF16])
def test_fused_at_a_scale_above_64(precision):
    """The fused call with the softmax relative to each sample's largest logit (s = 128), one-kernel
    form: same bits as the two calls for loss and feature gradient, centers and momentum equal
    up to the summation order, and the loss inside the bar against the oracle."""
    torch = _torch()
    N, B, D, r, s, m, lr, mu = 400_000, 200, 512, 0.1, 128.0, 0.5, 0.1, 0.9
    rng = np.random.default_rng(91)
    W0 = (rng.standard_normal((N, D)) * 0.01).astype(np.float32)
    X = rng.standard_normal((B, D)).astype(np.float32)
    labels = rng.integers(0, N, size=B).astype(np.int64)
    out = {}
    for fused in (False, True):
        _say("fused at s = 128", precision, "fused" if fused else "split")
        ctx = binding.Context(N, D, B, r, precision)
        Wd = torch.from_numpy(W0).cuda()
        vd = torch.zeros_like(Wd)
        cap = binding.pfc_num_sampled(N, B, r)
        idx = torch.zeros(cap, dtype=torch.int32, device="cuda")
        yl = torch.zeros(B, dtype=torch.int32, device="cuda")
        loss = torch.zeros(1, device="cuda")
        dX = torch.zeros(B, D, device="cuda")
        Xd, ld = torch.from_numpy(X).cuda(), torch.from_numpy(labels).cuda()
        k = ctx.pfc_sample(ld, r, 0, 0, idx, yl)
        if fused:
            ctx.pfc_forward_backward_update(Xd, Wd, vd, idx, k, yl, s, m, lr, mu, loss, dX)
        else:
            dW = torch.zeros(cap, D, device="cuda")
            ctx.pfc_forward_backward(Xd, Wd, idx, k, yl, s, m, loss, dX, dW)
            ctx.pfc_update(Wd, vd, idx, k, dW, lr, mu)
        torch.cuda.synchronize()
        assert ctx.pfc_check() == binding.PFC_OK
        out[fused] = (Wd.cpu().numpy(), vd.cpu().numpy(), float(loss.item()), dX.cpu().numpy(),
                      idx[:k].cpu().numpy(), yl.cpu().numpy())
        ctx.close()
    Wa, va, la, dXa, ia, ya = out[False]
    Wb, vb, lb, dXb, ib, yb = out[True]
    assert la == lb and dXa.tobytes() == dXb.tobytes() and np.array_equal(ia, ib)
    sel = ia.astype(np.int64)
    nrm = np.linalg.norm(Wa[sel].astype(np.float64), axis=1)
    assert row_rel_err(Wb[sel], Wa[sel], nrm) <= 1e-6
    assert rel_max(vb[sel], va[sel]) <= 1e-5
    o = O.forward_backward(X, W0[sel], ya, s, m)
    assert abs(lb - o["loss"]) <= LOSS_TOL[precision] * abs(o["loss"]), (lb, o["loss"])
    W64, v64 = W0.astype(np.float64), np.zeros((N, D))
    O.update(W64, v64, sel, o["dW"], lr, mu)
    err = row_rel_err(Wb[sel], W64[sel], np.linalg.norm(W64[sel], axis=1))
    _say("   loss", lb, o["loss"], "W row err", err)
    assert err <= W_TOL * 2      # the logit error, and with it the step of a center, doubles with s


def test_fused_tiny_workload_step():
    _run_steps(workloads.CONFIGS["tiny"], 1, fused=True)


def test_fused_medium_workload_ten_steps():
    _run_steps(workloads.CONFIGS["medium"], 10, fused=True)


def test_fused_large_workload_ten_steps():
    # 36,024 sampled classes: the one-kernel form, with a last round of half-height tiles
    _run_steps(workloads.CONFIGS["large"], 10, fused=True)


def test_fused_einval():
    torch = _torch()
    N, B, D = 2000, 64, 512
    ctx = binding.Context(N, D, B, 0.1, binding.PRECISION_FP32)
    W = torch.zeros(N, D, device="cuda")
    v = torch.zeros(N, D, device="cuda")
    X = torch.zeros(B, D, device="cuda")
    idx = torch.arange(200, dtype=torch.int32, device="cuda")
    yl = torch.zeros(B, dtype=torch.int32, device="cuda")
    loss = torch.zeros(1, device="cuda")
    dX = torch.zeros(B, D, device="cuda")
    good = dict(s=64.0, m=0.5, lr=0.1, mu=0.9)
    for bad in (dict(s=1e6), dict(s=0.0), dict(m=-0.1), dict(lr=float("nan")), dict(mu=float("nan"))):
        kw = dict(good, **bad)
        with pytest.raises(binding.PfcError):
            ctx.pfc_forward_backward_update(X, W, v, idx, 200, yl, kw["s"], kw["m"], kw["lr"],
                                            kw["mu"], loss, dX)
    with pytest.raises(binding.PfcError):
        ctx.pfc_forward_backward_update(X, W, v, idx, 0, yl, 64.0, 0.5, 0.1, 0.9, loss, dX)
    with pytest.raises(binding.PfcError):
        ctx.pfc_forward_backward_update(X, W, v, idx, 200, yl, 64.0, 0.5, 0.1, 0.9, loss, dX,
                                        margin_type=7)
    ctx.close()


@pytest.mark.parametrize("name,r", FULL_SIZE)
def test_fused_full_size_step(name, r):
    """One fused step at the full class count against the oracle run on the sampled rows."""
    torch = _torch()
    wl = workloads.CONFIGS[name].with_(r=r)
    Wd = _device_weight(wl)
    W_before = _weight_cache[(wl.cfg_id, wl.N, wl.D)]     # the pristine copy (never written)
    vd = torch.zeros_like(Wd)
    ctx = binding.Context(wl.N, wl.D, wl.B, wl.r, wl.precision)
    cap = binding.pfc_num_sampled(wl.N, wl.B, wl.r)
    idx_d = torch.zeros(cap, dtype=torch.int32, device="cuda")
    yl_d = torch.zeros(wl.B, dtype=torch.int32, device="cuda")
    loss_d = torch.zeros(1, device="cuda")
    dX_d = torch.zeros(wl.B, wl.D, device="cuda")
    X = workloads.make_features(wl, 0)
    labels = workloads.make_labels(wl, 0)
    labels_d = torch.from_numpy(labels).cuda()
    X_d = torch.from_numpy(X).cuda()
    _say("fused full size step", name, r)
    k = ctx.pfc_sample(labels_d, wl.r, wl.seed, 0, idx_d, yl_d)
    ctx.pfc_forward_backward_update(X_d, Wd, vd, idx_d, k, yl_d, wl.s, wl.m, wl.lr, wl.mu, loss_d,
                                    dX_d)
    torch.cuda.synchronize()
    assert ctx.pfc_check() == binding.PFC_OK
    oidx, oyl, ok = O.sample(labels, wl.N, wl.r, wl.seed, 0)
    assert k == ok and np.array_equal(idx_d[:k].cpu().numpy(), oidx)
    sel = torch.from_numpy(oidx.astype(np.int64)).cuda()
    W_S = W_before[sel].cpu().numpy()
    o = O.forward_backward(X, W_S, oyl, wl.s, wl.m)
    gl = float(loss_d.item())
    assert abs(gl - o["loss"]) <= LOSS_TOL[wl.precision] * abs(o["loss"])
    assert rel_max(dX_d.cpu().numpy(), o["dX"]) <= GRAD_TOL[wl.precision]
    W_S64 = W_S.astype(np.float64)
    v_S64 = np.zeros_like(W_S64)
    O.update(W_S64, v_S64, np.arange(k), o["dW"], wl.lr, wl.mu)
    err = row_rel_err(Wd[sel].cpu().numpy(), W_S64, np.linalg.norm(W_S64, axis=1))
    _say("   loss", gl, o["loss"], "W row err", err)
    assert err <= W_TOL
    v_g = vd[sel].cpu().numpy()
    assert rel_max(v_g, v_S64) <= GRAD_TOL[wl.precision]
    rx, _ = row_rel_max(dX_d.cpu().numpy(), o["dX"])
    rv, nv = row_rel_max(v_g, v_S64)
    _say("   per-row err dX", rx, "v", rv, "rows", nv, "of", k)
    assert rx <= ROW_GRAD_TOL[wl.precision] and rv <= ROW_GRAD_TOL[wl.precision]
    assert nv >= 0.9 * k
    del o, v_g
    mask = torch.ones(wl.N, dtype=torch.bool, device="cuda")
    mask[sel] = False
    same = (Wd.view(torch.int32) == W_before.view(torch.int32)).all(dim=1)
    assert bool(same[mask].all())
    assert not bool(vd[mask].any())
    assert not bool(same[~mask].all())
    ctx.close()
