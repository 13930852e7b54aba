"""GPU parity of pfc_forward_backward / pfc_update / whole steps against the fp64 oracle.

Bars (stated by the benchmark spec): loss within 1e-5 relative (fp32 operands) or 2e-3 relative (bf16
operands); updated centers within 1e-3 max-abs relative to the row norm.  Gradient bars are this
repository's own: against the largest entry of the whole matrix 2e-5 (fp32 operands) and 1e-2
(bf16 operands, 2^-9 relative rounding each), and row by row against each row's own largest
entry 1e-4 / 5e-2 (pfc_harness.ROW_GRAD_TOL), which is the check that constrains the rows of
centers that are nobody's label.
"""
import sys

import numpy as np
import pytest

from oracle import pfc_oracle as O
from paper_2203_15565_amd import binding, workloads
from pfc_harness import (ROW_GRAD_TOL, dim_amp, gpu_forward_backward, gpu_sample, rel_max,
                         row_rel_err, row_rel_max)

pytestmark = pytest.mark.gpu

LOSS_TOL = {binding.PRECISION_FP32: 1e-5, binding.PRECISION_BF16: 2e-3}
GRAD_TOL = {binding.PRECISION_FP32: 2e-5, binding.PRECISION_BF16: 1e-2}
W_TOL = 1e-3


def _say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _torch():
    import torch
    return torch


def _case(N, B, D, k_r, seed, wscale=0.01):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((B, D)).astype(np.float32)
    W = (rng.standard_normal((N, D)) * wscale).astype(np.float32)
    labels = rng.integers(0, N, size=B)
    return X, W, labels


def _fb_parity(precision, N, B, D, r, s, m, seed, wscale=0.01, dup=False):
    torch = _torch()
    X, W, labels = _case(N, B, D, r, seed, wscale)
    if dup:
        labels[: B // 2] = labels[0]
    ctx = binding.Context(N, D, B, r, precision)
    idx, yl, k = gpu_sample(ctx, labels, r, 0, 0)
    idx = idx[:k]
    Wd = torch.from_numpy(W).cuda()
    _say("fb_parity", precision, N, B, D, r, s, m, "k", k)
    loss, dX, dWn = gpu_forward_backward(ctx, X, Wd, idx, yl, s, m)
    assert ctx.pfc_check() == binding.PFC_OK
    o = O.forward_backward(X, W[idx.astype(np.int64)], yl, s, m)
    assert abs(loss - o["loss"]) <= LOSS_TOL[precision] * abs(o["loss"]), (loss, o["loss"])
    assert np.isfinite(dX).all() and np.isfinite(dWn).all()
    ex = rel_max(dX, o["dX"])
    ew = rel_max(dWn, o["dWn"])
    rx, _ = row_rel_max(dX, o["dX"])
    rw, nrows = row_rel_max(dWn, o["dWn"])
    _say("   loss", loss, o["loss"], "dX err", ex, "dWn err", ew, "per row: dX", rx, "dWn", rw,
         "rows", nrows, "of", k)
    # the error of a logit is s * (error of the cosine), which grows for short rows
    amp = max(1.0, s / 64.0) * dim_amp(precision, D)
    assert ex <= GRAD_TOL[precision] * amp, ex
    assert ew <= GRAD_TOL[precision] * amp, ew
    assert rx <= ROW_GRAD_TOL[precision] * amp, rx
    assert rw <= ROW_GRAD_TOL[precision] * amp, rw
    # (at large scales the softmax is so peaked that many rows fall below the floor of the row bar)
    assert nrows >= (0.9 if s <= 64.0 else 0.5) * k
    # second call on the same context and inputs: bit-identical outputs
    loss2, dX2, dWn2 = gpu_forward_backward(ctx, X, Wd, idx, yl, s, m)
    assert loss2 == loss and dX2.tobytes() == dX.tobytes() and dWn2.tobytes() == dWn.tobytes()
    ctx.close()
    return o


@pytest.mark.parametrize("N,B,D,r", [(10_000, 128, 512, 0.1),     # the Tiny workload's shape
                                     (3000, 100, 256, 0.1),       # ragged B and k (300)
                                     (5000, 37, 1024, 0.13),      # k = 650, odd B
                                     (700, 130, 768, 1.0),        # r = 1: full FC, k = 700
                                     # D a multiple of 64 but not of 256 (rows padded inside)
                                     (3000, 100, 64, 0.1), (2500, 70, 192, 0.2),
                                     (4000, 96, 320, 0.1), (3000, 50, 960, 0.1)])
def test_forward_backward_fp32(N, B, D, r):
    _fb_parity(binding.PRECISION_FP32, N, B, D, r, 64.0, 0.5, seed=N + B)


@pytest.mark.parametrize("N,B,D,r", [(10_000, 128, 512, 0.1), (3000, 100, 256, 0.1),
                                     (20_000, 300, 512, 0.077), (700, 130, 768, 1.0),
                                     (3000, 100, 128, 0.1), (2500, 70, 448, 0.2),
                                     (4000, 300, 576, 0.1), (700, 40, 64, 1.0)])
def test_forward_backward_bf16(N, B, D, r):
    _fb_parity(binding.PRECISION_BF16, N, B, D, r, 64.0, 0.5, seed=N + B + 1)


@pytest.mark.parametrize("precision", [binding.PRECISION_FP32, binding.PRECISION_BF16])
def test_forward_backward_variants(precision):
    # m = 0 (plain softmax CE), small scale, duplicated labels, unit-scale centers
    _fb_parity(precision, 4000, 64, 512, 0.1, 64.0, 0.0, seed=11)
    _fb_parity(precision, 4000, 64, 512, 0.1, 16.0, 0.35, seed=12, wscale=1.0)
    _fb_parity(precision, 4000, 96, 512, 0.1, 64.0, 0.5, seed=13, dup=True)


@pytest.mark.parametrize("precision", [binding.PRECISION_FP32, binding.PRECISION_BF16])
def test_forward_backward_large_scale(precision):
    """Scales above 64: exp(z) would leave the fp32 range, the softmax runs relative to each
    sample's largest logit (found by one more pass of the logit GEMM)."""
    _fb_parity(precision, 10_000, 128, 512, 0.1, 128.0, 0.5, seed=31)
    _fb_parity(precision, 3000, 100, 256, 0.1, 200.0, 0.3, seed=32)
    # unit-scale centers close to the features' scale: cosines up to ~0.2, logits spread over 80
    _fb_parity(precision, 4000, 96, 512, 0.1, 400.0, 0.5, seed=33, dup=True)


@pytest.mark.parametrize("precision", [binding.PRECISION_FP32, binding.PRECISION_BF16])
def test_forward_backward_batch_of_several_label_windows(precision):
    """Batches above 1024 samples: the label part of the center gradient is summed per window of
    1024 samples and the window sums are combined; half of the batch carries one label here, so
    that class has a sum in every window."""
    _fb_parity(precision, 20_000, 2500, 512, 0.05, 64.0, 0.5, seed=41, dup=True)
    _fb_parity(precision, 20_000, 3072, 256, 0.05, 64.0, 0.5, seed=42)
    # 8192 samples, eight windows, most classes in several of them
    _fb_parity(precision, 3000, 8192, 256, 0.1, 64.0, 0.5, seed=43)


@pytest.mark.parametrize("precision", [binding.PRECISION_FP32, binding.PRECISION_BF16])
def test_forward_backward_smallest_shapes(precision):
    """One sample; two classes; the shortest rows."""
    _fb_parity(precision, 5, 1, 64, 1.0, 64.0, 0.5, seed=51)
    _fb_parity(precision, 2, 1, 512, 1.0, 64.0, 0.5, seed=52)
    _fb_parity(precision, 2, 3, 128, 1.0, 16.0, 0.2, seed=53)


@pytest.mark.parametrize("precision", [binding.PRECISION_FP32, binding.PRECISION_BF16])
def test_one_class_only(precision):
    """N = 1: the softmax runs over the label alone, so the loss and every gradient are zero
    whatever the margin makes of the logit (Eq. 1 with a single term)."""
    torch = _torch()
    N, B, D = 1, 3, 256
    rng = np.random.default_rng(54)
    X = rng.standard_normal((B, D)).astype(np.float32)
    W = rng.standard_normal((N, D)).astype(np.float32)
    labels = np.zeros(B, dtype=np.int64)
    ctx = binding.Context(N, D, B, 1.0, precision)
    idx, yl, k = gpu_sample(ctx, labels, 1.0, 0, 0)
    assert k == 1 and idx[0] == 0 and not yl.any()
    _say("one class", precision)
    loss, dX, dWn = gpu_forward_backward(ctx, X, torch.from_numpy(W).cuda(), idx[:k], yl, 64.0, 0.5)
    o = O.forward_backward(X, W, yl, 64.0, 0.5)
    assert abs(o["loss"]) < 1e-12 and abs(loss) < 1e-5
    assert np.abs(dX).max() < 1e-5 and np.abs(dWn[:k]).max() < 1e-5
    ctx.close()


def test_forward_backward_minimum_k():
    """k = U (no negatives outside the batch), including k far below one tile."""
    _fb_parity(binding.PRECISION_FP32, 100_000, 24, 512, 1e-5, 64.0, 0.5, seed=14)
    _fb_parity(binding.PRECISION_BF16, 100_000, 24, 512, 1e-5, 64.0, 0.5, seed=15)


def test_forward_backward_einval():
    torch = _torch()
    ctx = binding.Context(1000, 512, 8, 0.1, binding.PRECISION_FP32)
    X = torch.zeros(8, 512, device="cuda")
    W = torch.zeros(1000, 512, device="cuda")
    idx = torch.arange(100, dtype=torch.int32, device="cuda")
    yl = torch.zeros(8, dtype=torch.int32, device="cuda")
    loss = torch.zeros(1, device="cuda")
    dX = torch.zeros(8, 512, device="cuda")
    dW = torch.zeros(100, 512, device="cuda")
    for kw in (dict(k=0), dict(k=101), dict(s=1e6), dict(s=0.0), dict(m=-0.1), dict(m=3.2)):
        args = dict(k=100, s=64.0, m=0.5)
        args.update(kw)
        with pytest.raises(binding.PfcError) as e:
            ctx.pfc_forward_backward(X, W, idx, args["k"], yl, args["s"], args["m"], loss, dX, dW)
        assert e.value.code == binding.PFC_EINVAL
    # out-of-range local label / index is recorded, not a fault
    yl[3] = 100
    ctx.pfc_forward_backward(X, W, idx, 100, yl, 64.0, 0.5, loss, dX, dW)
    assert ctx.pfc_check() == binding.PFC_ELABEL
    yl[3] = 0
    idx[7] = 1000
    ctx.pfc_forward_backward(X, W, idx, 100, yl, 64.0, 0.5, loss, dX, dW)
    assert ctx.pfc_check() == binding.PFC_ELABEL
    ctx.close()


@pytest.mark.parametrize("D", [512, 64, 448, 1024])
def test_update_parity_and_untouched_rows(D):
    torch = _torch()
    N, k = 5000, 700
    rng = np.random.default_rng(21)
    W = (rng.standard_normal((N, D)) * 0.01).astype(np.float32)
    v = (rng.standard_normal((N, D)) * 0.001).astype(np.float32)
    idx = np.sort(rng.choice(N, size=k, replace=False)).astype(np.int32)
    g = rng.standard_normal((k, D)).astype(np.float32)
    ctx = binding.Context(N, D, 8, 0.2, binding.PRECISION_FP32)
    Wd, vd = torch.from_numpy(W).cuda(), torch.from_numpy(v).cuda()
    _say("update parity")
    ctx.pfc_update(Wd, vd, torch.from_numpy(idx).cuda(), k, torch.from_numpy(g).cuda(), 0.1, 0.9)
    torch.cuda.synchronize()
    W1, v1 = Wd.cpu().numpy(), vd.cpu().numpy()
    # oracle: the entry point takes dL/d wn and applies the normalisation Jacobian itself
    W64, v64 = W.astype(np.float64), v.astype(np.float64)
    rows = W64[idx]
    nrm = np.linalg.norm(rows, axis=1, keepdims=True)
    wn = rows / nrm
    dW = (g - (g * wn).sum(axis=1, keepdims=True) * wn) / nrm
    O.update(W64, v64, idx, dW, 0.1, 0.9)
    rest = np.setdiff1d(np.arange(N), idx)
    assert W1[rest].tobytes() == W[rest].tobytes()
    assert v1[rest].tobytes() == v[rest].tobytes()
    assert rel_max(v1[idx], v64[idx]) < 1e-5
    assert row_rel_err(W1[idx], W64[idx], np.linalg.norm(W64[idx], axis=1)) < 1e-5
    ctx.close()


def _run_steps(wl, nsteps, check_every_step=True, fused=False):
    """Whole steps sample -> forward/backward -> update on the GPU next to the oracle
    (fused: forward/backward and update in the one call pfc_forward_backward_update)."""
    torch = _torch()
    W0 = workloads.make_weight(wl)
    W64, v64 = W0.astype(np.float64), np.zeros(W0.shape)
    Wd = torch.from_numpy(W0).cuda()
    vd = torch.zeros_like(Wd)
    ctx = binding.Context(wl.N, wl.D, wl.B, wl.r, wl.precision)
    cap = binding.pfc_num_sampled(wl.N, wl.B, wl.r)
    idx_d = torch.zeros(cap, dtype=torch.int32, device="cuda")
    yl_d = torch.zeros(wl.B, dtype=torch.int32, device="cuda")
    loss_d = torch.zeros(1, device="cuda")
    dX_d = torch.zeros(wl.B, wl.D, device="cuda")
    dW_d = torch.zeros(cap, wl.D, device="cuda")
    touched = np.zeros(wl.N, dtype=bool)
    err = 0.0        # largest row error of the centers seen so far
    for t in range(nsteps):
        X = workloads.make_features(wl, t)
        labels = workloads.make_labels(wl, t)
        _say("step", wl.name, t)
        labels_d = torch.from_numpy(labels).cuda()      # referenced until the synchronize below
        X_d = torch.from_numpy(X).cuda()
        k = ctx.pfc_sample(labels_d, wl.r, wl.seed, t, idx_d, yl_d)
        if fused:
            ctx.pfc_forward_backward_update(X_d, Wd, vd, idx_d, k, yl_d, wl.s, wl.m, wl.lr, wl.mu,
                                            loss_d, dX_d)
        else:
            ctx.pfc_forward_backward(X_d, Wd, idx_d, k, yl_d, wl.s, wl.m, loss_d, dX_d, dW_d)
            ctx.pfc_update(Wd, vd, idx_d, k, dW_d, wl.lr, wl.mu)
        torch.cuda.synchronize()
        assert ctx.pfc_check() == binding.PFC_OK
        oloss, odX, oidx, oyl, fb = O.step(X, labels, W64, v64, r=wl.r, s=wl.s, m=wl.m, lr=wl.lr,
                                           mu=wl.mu, seed=wl.seed, step=t)
        assert np.array_equal(idx_d[:k].cpu().numpy(), oidx)
        assert np.array_equal(yl_d.cpu().numpy(), oyl)
        touched[oidx] = True
        gl = float(loss_d.item())
        assert abs(gl - oloss) <= LOSS_TOL[wl.precision] * abs(oloss), (t, gl, oloss)
        assert rel_max(dX_d.cpu().numpy(), odX) <= GRAD_TOL[wl.precision] * dim_amp(wl.precision, wl.D)
        # row by row; centers that have drifted by `err` of their norm move the logits by s * err
        row_tol = ROW_GRAD_TOL[wl.precision] * dim_amp(wl.precision, wl.D) + wl.s * err
        assert row_rel_max(dX_d.cpu().numpy(), odX)[0] <= row_tol
        if not fused:
            rw, nrows = row_rel_max(dW_d[:k].cpu().numpy(), fb["dWn"])
            assert rw <= row_tol and nrows >= 0.9 * k, (t, rw, nrows)
        if check_every_step or t == nsteps - 1:
            Wg = Wd.cpu().numpy()
            sel = oidx.astype(np.int64)
            err = max(err, row_rel_err(Wg[sel], W64[sel], np.linalg.norm(W64[sel], axis=1)))
            _say("   loss", gl, oloss, "W row err so far", err)
            assert err <= W_TOL, (t, err)
    Wg, vg = Wd.cpu().numpy(), vd.cpu().numpy()
    assert Wg[~touched].tobytes() == W0[~touched].tobytes()       # never-sampled rows: bit-exact
    assert not vg[~touched].any()
    tsel = np.nonzero(touched)[0]
    err = max(err, row_rel_err(Wg[tsel], W64[tsel], np.linalg.norm(W64[tsel], axis=1)))
    assert err <= W_TOL, err
    # momentum of every row ever sampled, row by row against its own largest entry.  After several
    # steps the two sides no longer multiply the same centers: a center off by `err` of its norm
    # moves its logits by up to s * err, and a row's gradient by as much (relative).
    rv, nv = row_rel_max(vg[tsel], v64[tsel])
    _say("   v per-row err", rv, "rows", nv, "of", tsel.size)
    assert rv <= (ROW_GRAD_TOL[wl.precision] * dim_amp(wl.precision, wl.D) +
                  (wl.s * err if nsteps > 1 else 0.0)), (rv, err)
    assert nv >= 0.9 * tsel.size
    ctx.close()


def test_tiny_workload_step():
    _run_steps(workloads.CONFIGS["tiny"], 1)


@pytest.mark.parametrize("D,precision", [(128, binding.PRECISION_FP32), (320, binding.PRECISION_BF16)])
@pytest.mark.parametrize("fused", [False, True])
def test_steps_with_other_row_lengths(D, precision, fused):
    """Three whole steps with D a multiple of 64 that is not one of 256: both call sequences."""
    # (B as in the Medium workload: the bar on the updated centers is relative to their norm, and
    # how far a label center moves in a step, in units of its norm, goes as 1/B)
    wl = workloads.CONFIGS["tiny"].with_(name="tiny-D%d" % D, D=D, N=20_000, B=512,
                                         precision=precision)
    _run_steps(wl, 3, fused=fused)


def test_medium_workload_ten_steps():
    _run_steps(workloads.CONFIGS["medium"], 10)


def test_large_workload_ten_steps():
    _run_steps(workloads.CONFIGS["large"], 10)


_weight_cache: dict = {}


def _device_weight(wl):
    """The workload's initial centers on the device, uploaded chunk by chunk (the host never holds
    all of W).  The pristine copy of the last workload asked for stays on the device, so that the
    tests of one workload do not draw its 1e9 normal deviates again each; callers get a clone."""
    torch = _torch()
    key = (wl.cfg_id, wl.N, wl.D)
    if key not in _weight_cache:
        _weight_cache.clear()
        torch.cuda.empty_cache()
        Wd = torch.empty((wl.N, wl.D), dtype=torch.float32, device="cuda")
        for row0, chunk in workloads.weight_chunks(wl):
            Wd[row0:row0 + chunk.shape[0]].copy_(torch.from_numpy(chunk))
        _weight_cache[key] = Wd
    return _weight_cache[key].clone()


# every ratio of the headline sweep, the full-FC run of the large workload (r = 1, "FC-1.0" in
# Tab. 1), the 10M-class workload and the two enlarged batches without extra negatives (Tab. 7)
FULL_SIZE = [("headline", 0.05), ("headline", 0.1), ("headline", 0.2), ("headline", 0.4),
             ("ultrafast8k", 1e-9), ("ultrafast16k", 1e-9), ("large", 1.0), ("extreme", 0.05)]


@pytest.mark.parametrize("name,r", FULL_SIZE)
def test_full_size_step(name, r):
    """One whole step at the full class count, in the launch configuration bench.py times.
    The oracle runs on the sampled rows W[idx] only (the method never reads the others); rows
    outside idx are compared bit for bit on the device."""
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
    dW_d = torch.zeros(cap, wl.D, device="cuda")
    X = workloads.make_features(wl, 0)
    labels = workloads.make_labels(wl, 0)
    labels_d = torch.from_numpy(labels).cuda()
    X_d = torch.from_numpy(X).cuda()
    _say("full size step", name, r)
    k = ctx.pfc_sample(labels_d, wl.r, wl.seed, 0, idx_d, yl_d)
    ctx.pfc_forward_backward(X_d, Wd, idx_d, k, yl_d, wl.s, wl.m, loss_d, dX_d, dW_d)
    torch.cuda.synchronize()
    dWn_g = dW_d[:k].cpu().numpy()
    ctx.pfc_update(Wd, vd, idx_d, k, dW_d, wl.lr, wl.mu)
    torch.cuda.synchronize()
    assert ctx.pfc_check() == binding.PFC_OK

    oidx, oyl, ok = O.sample(labels, wl.N, wl.r, wl.seed, 0)
    assert k == ok and np.array_equal(idx_d[:k].cpu().numpy(), oidx)
    assert np.array_equal(yl_d.cpu().numpy(), oyl)
    sel = torch.from_numpy(oidx.astype(np.int64)).cuda()
    W_S = W_before[sel].cpu().numpy()
    o = O.forward_backward(X, W_S, oyl, wl.s, wl.m)
    gl = float(loss_d.item())
    _say("   loss", gl, o["loss"])
    assert abs(gl - o["loss"]) <= LOSS_TOL[wl.precision] * abs(o["loss"])
    assert rel_max(dX_d.cpu().numpy(), o["dX"]) <= GRAD_TOL[wl.precision]
    assert rel_max(dWn_g, o["dWn"]) <= GRAD_TOL[wl.precision]
    rx, _ = row_rel_max(dX_d.cpu().numpy(), o["dX"])
    rw, nrows = row_rel_max(dWn_g, o["dWn"])
    _say("   per-row err dX", rx, "dWn", rw, "rows", nrows, "of", k)
    assert rx <= ROW_GRAD_TOL[wl.precision] and rw <= ROW_GRAD_TOL[wl.precision]
    assert nrows >= 0.9 * k
    # positive rows separately: their gradient is dominated by the fp32 label column
    prow = np.unique(oyl)
    assert rel_max(dWn_g[prow], o["dWn"][prow]) <= 1e-3
    W_S64 = W_S.astype(np.float64)
    v_S64 = np.zeros_like(W_S64)
    O.update(W_S64, v_S64, np.arange(k), o["dW"], wl.lr, wl.mu)
    err = row_rel_err(Wd[sel].cpu().numpy(), W_S64, np.linalg.norm(W_S64, axis=1))
    _say("   W row err", err)
    assert err <= W_TOL
    v_g = vd[sel].cpu().numpy()
    assert rel_max(v_g, v_S64) <= GRAD_TOL[wl.precision]
    rv, nv = row_rel_max(v_g, v_S64)
    _say("   per-row err v", rv)
    assert rv <= ROW_GRAD_TOL[wl.precision] and nv >= 0.9 * k
    del o, v_g, dWn_g
    # unsampled rows: bit-identical W, untouched (zero) v -- checked on the device
    mask = torch.ones(wl.N, dtype=torch.bool, device="cuda")
    mask[sel] = False
    same = (Wd.view(torch.int32) == W_before.view(torch.int32)).all(dim=1)
    assert bool(same[mask].all())
    assert not bool(vd[mask].any())
    assert not bool(same[~mask].all())       # and the sampled rows did move
    ctx.close()


@pytest.mark.parametrize("fused", [False, True])
def test_replay_from_saved_state_is_bit_identical(fused):
    """Resume: step t replayed from a saved (W, v) with the same (seed, step) in a NEW context gives
    bit-identical W, v, loss and feature gradient (sampling is a pure function of seed, step and
    labels; no kernel uses floating-point atomics)."""
    torch = _torch()
    wl = workloads.CONFIGS["medium"].with_(N=340_000)     # enough classes for the one-kernel fused form
    rng = np.random.default_rng(99)
    W0 = (rng.standard_normal((wl.N, wl.D)) * 0.01).astype(np.float32)

    def run(ctx, Wd, vd, t):
        cap = binding.pfc_num_sampled(wl.N, wl.B, wl.r)
        idx = torch.zeros(cap, dtype=torch.int32, device="cuda")
        yl = torch.zeros(wl.B, dtype=torch.int32, device="cuda")
        loss = torch.zeros(1, device="cuda")
        dX = torch.zeros(wl.B, wl.D, device="cuda")
        X = torch.from_numpy(workloads.make_features(wl, t)).cuda()
        lab = torch.from_numpy(workloads.make_labels(wl, t)).cuda()
        k = ctx.pfc_sample(lab, wl.r, wl.seed, t, idx, yl)
        if fused:
            ctx.pfc_forward_backward_update(X, Wd, vd, idx, k, yl, wl.s, wl.m, wl.lr, wl.mu, loss, dX)
        else:
            dW = torch.zeros(cap, wl.D, device="cuda")
            ctx.pfc_forward_backward(X, Wd, idx, k, yl, wl.s, wl.m, loss, dX, dW)
            ctx.pfc_update(Wd, vd, idx, k, dW, wl.lr, wl.mu)
        torch.cuda.synchronize()
        assert ctx.pfc_check() == binding.PFC_OK
        return float(loss.item()), dX.cpu().numpy().tobytes()

    _say("replay", "fused" if fused else "three calls")
    a = binding.Context(wl.N, wl.D, wl.B, wl.r, wl.precision)
    Wd = torch.from_numpy(W0).cuda()
    vd = torch.zeros_like(Wd)
    for t in range(2):
        run(a, Wd, vd, t)
    W_saved, v_saved = Wd.clone(), vd.clone()             # the checkpoint after step 1
    ref = run(a, Wd, vd, 2)
    b = binding.Context(wl.N, wl.D, wl.B, wl.r, wl.precision)
    W2, v2 = W_saved.clone(), v_saved.clone()
    got = run(b, W2, v2, 2)
    assert got == ref
    assert torch.equal(W2.view(torch.int32), Wd.view(torch.int32))
    assert torch.equal(v2.view(torch.int32), vd.view(torch.int32))
    assert not torch.equal(W2, W_saved)
    a.close()
    b.close()


@pytest.mark.parametrize("precision", [binding.PRECISION_FP32, binding.PRECISION_BF16])
def test_features_parallel_to_centers(precision):
    """Degenerate cosines: some features are exact multiples of a sampled center (cosine +1 with
    it) or of a negated center (cosine -1), for label and non-label centers alike: the clamp, and
    the margin derivative sin(theta + m)/sin(theta) at sin(theta) = 0, where the reading with the
    floor of 1e-12 under the root makes it 4.8e5.  Loss, every output finite, and all gradients and
    updated centers that do not involve a sample parallel to its OWN label center stay inside the
    bars; for those samples (and their label centers) the gradient along the common direction is
    5e5 times the usual size and its projection is the rounding residue of whatever precision
    computed it, so nothing but finiteness is asserted about them."""
    torch = _torch()
    N, B, D, r, s, m = 6000, 96, 512, 0.1, 64.0, 0.5
    rng = np.random.default_rng(55)
    X = rng.standard_normal((B, D)).astype(np.float32)
    W = (rng.standard_normal((N, D)) * 0.01).astype(np.float32)
    labels = rng.permutation(N)[:B]       # distinct labels: one sample per label center
    X[0] = 37.0 * W[labels[0]]            # cosine +1 with its own label center
    X[1] = -5.0 * W[labels[1]]            # cosine -1 with its own label center
    X[2] = 11.0 * W[labels[3]]            # cosine +1 with another sample's label center
    X[4] = -2.0 * W[labels[5]]            # cosine -1 with another sample's label center
    own = np.array([0, 1])                # samples parallel to their own label center
    ctx = binding.Context(N, D, B, r, precision)
    idx, yl, k = gpu_sample(ctx, labels, r, 0, 0)
    idx = idx[:k]
    Wd = torch.from_numpy(W).cuda()
    vd = torch.zeros_like(Wd)
    _say("degenerate cosines", precision)
    loss, dX, dWn = gpu_forward_backward(ctx, X, Wd, idx, yl, s, m)
    idx_d = torch.from_numpy(idx).cuda()
    ctx.pfc_update(Wd, vd, idx_d, k, torch.from_numpy(dWn).cuda(), 0.1, 0.9)
    torch.cuda.synchronize()
    assert ctx.pfc_check() == binding.PFC_OK
    sel = idx.astype(np.int64)
    o = O.forward_backward(X, W[sel], yl, s, m)
    assert abs(o["cos"]).max() == 1.0                       # the case is what it claims to be
    Wg, vg = Wd.cpu().numpy(), vd.cpu().numpy()
    assert np.isfinite(dX).all() and np.isfinite(dWn).all() and np.isfinite(loss)
    assert np.isfinite(Wg).all() and np.isfinite(vg).all()
    assert abs(loss - o["loss"]) <= LOSS_TOL[precision] * abs(o["loss"]), (loss, o["loss"])
    ok_s = np.setdiff1d(np.arange(B), own)                  # samples
    ok_c = np.setdiff1d(np.arange(k), yl[own])              # positions in the sampled set
    assert rel_max(dX[ok_s], o["dX"][ok_s]) <= GRAD_TOL[precision]
    assert rel_max(dWn[ok_c], o["dWn"][ok_c]) <= GRAD_TOL[precision]
    W64, v64 = W.astype(np.float64), np.zeros((N, D))
    O.update(W64, v64, sel, o["dW"], 0.1, 0.9)
    rows = sel[ok_c]
    err = row_rel_err(Wg[rows], W64[rows], np.linalg.norm(W64[rows], axis=1))
    _say("   loss", loss, o["loss"], "W row err", err)
    assert err <= W_TOL
    assert rel_max(vg[rows], v64[rows]) <= GRAD_TOL[precision]
    rest = np.setdiff1d(np.arange(N), sel)
    assert Wg[rest].tobytes() == W[rest].tobytes() and not vg[rest].any()
    ctx.close()


@pytest.mark.parametrize("fused", [False, True])
def test_step_under_graph_capture(fused):
    """A whole step recorded into a HIP graph (the library allocates nothing, records no memset and
    never waits for the GPU when ceil(r N) >= B) and replayed several times, with eager work and
    synchronisations in between: every replay from a given (W, v) gives the bits of the eager step."""
    torch = _torch()
    wl = workloads.CONFIGS["medium"].with_(N=340_000 if fused else 93_431)
    rng = np.random.default_rng(7)
    W0 = torch.from_numpy((rng.standard_normal((wl.N, wl.D)) * 0.01).astype(np.float32)).cuda()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        ctx = binding.Context(wl.N, wl.D, wl.B, wl.r, wl.precision)
        cap = binding.pfc_num_sampled(wl.N, wl.B, wl.r)
        idx = torch.zeros(cap, dtype=torch.int32, device="cuda")
        yl = torch.zeros(wl.B, dtype=torch.int32, device="cuda")
        loss = torch.zeros(1, device="cuda")
        dX = torch.zeros(wl.B, wl.D, device="cuda")
        dW = torch.zeros(cap, wl.D, device="cuda")
        X = torch.from_numpy(workloads.make_features(wl, 0)).cuda()
        lab = torch.from_numpy(workloads.make_labels(wl, 0)).cuda()
        Wd, vd = W0.clone(), torch.zeros_like(W0)

        def step():
            k = ctx.pfc_sample(lab, wl.r, wl.seed, 0, idx, yl)
            if fused:
                ctx.pfc_forward_backward_update(X, Wd, vd, idx, k, yl, wl.s, wl.m, wl.lr, wl.mu,
                                                loss, dX)
            else:
                ctx.pfc_forward_backward(X, Wd, idx, k, yl, wl.s, wl.m, loss, dX, dW)
                ctx.pfc_update(Wd, vd, idx, k, dW, wl.lr, wl.mu)

        _say("graph capture", "fused" if fused else "three calls")
        step()                                   # eager: also raises the kernels' LDS limits
        stream.synchronize()
        Wd.copy_(W0)
        vd.zero_()
        step()
        stream.synchronize()
        ref = (Wd.clone(), vd.clone(), loss.clone(), dX.clone())
        graph = torch.cuda.CUDAGraph()
        Wd.copy_(W0)
        vd.zero_()
        with torch.cuda.graph(graph, stream=stream):
            step()
        for rep in range(3):
            Wd.copy_(W0)                         # eager work between the replays
            vd.zero_()
            loss.fill_(-1.0)
            stream.synchronize()
            graph.replay()
            stream.synchronize()
            for got, want in zip((Wd, vd, loss, dX), ref):
                assert torch.equal(got.view(torch.int32), want.view(torch.int32)), rep
        assert ctx.pfc_check() == binding.PFC_OK
        ctx.close()
