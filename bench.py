#!/usr/bin/env python3
"""Benchmark of one Partial FC training step (sample + forward/backward + update) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload headline] [--no-cpu-baseline]
                    [--fused]

Prints ONE JSON line: whole-step throughput in samples/s with all inputs resident in HBM, the
roofline of the dominant kernel (measured with HIP events on the library's stream) and the fp64
CPU oracle timed on the same workload as a reported baseline.  `value` is the sequence the metric
names, pfc_sample + pfc_forward_backward + pfc_update; the sequence with the one fused call
pfc_forward_backward_update is timed as well and reported as `value_fused_call` (--fused swaps
the two).  `calls_ms` holds the duration of every ABI call on its own.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, GB/s
PEAK_BF16_TFLOPS = 2500.0      # dense bf16 MFMA
PEAK_FP32_MFMA_TFLOPS = 157.3  # fp32 MFMA

# HBM bytes per launch (read + written) from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# summarised in profiles/headline_step_hbm_traffic.md, keyed by (workload, r, kernel).  None where
# no counter run has been recorded.
MEASURED_TRAFFIC_BYTES: dict = {
    ("headline", 0.1, "gemm_dweight_update"): 2171342916,
    ("headline", 0.1, "update"): 2115907072,
    ("headline", 0.1, "gather_normalize_w"): 636338241,
    ("headline", 0.1, "gemm_logits"): 723901584,
    ("headline", 0.1, "gemm_dweight"): 905431780,
    ("headline", 0.1, "gemm_dfeatures"): 700291405,
}

# Fraction of a GEMM kernel's own cycles in which an MFMA pipe was busy, from the rocprofv3 --pmc
# run summarised in profiles/headline_step_mfma_lds_counters.md (SQ_VALU_MFMA_BUSY_CYCLES over
# the kernel's SQ_BUSY_CYCLES: independent of the clock the kernel ran at).
MEASURED_MFMA_BUSY: dict = {
    ("headline", 0.1, "gemm_logits"): 0.352,
    ("headline", 0.1, "gemm_dweight"): 0.373,
    ("headline", 0.1, "gemm_dfeatures"): 0.591,
    ("headline", 0.1, "gemm_dweight_update"): 0.196,
}


def algorithmic_work(B: int, D: int, k: int, precision: int) -> dict:
    """Algorithmic flops / HBM bytes of the main kernels for one step (what the method must
    compute or move, not what this implementation adds)."""
    es = 2 if precision == 1 else 4
    gemm = 2.0 * B * D * k
    return {
        "gemm_logits": ("mfma", gemm),
        "gemm_dweight": ("mfma", gemm),
        "gemm_dfeatures": ("mfma", gemm),
        "gather_normalize_w": ("hbm", k * D * (4 + es) + 4.0 * k),
        "update": ("hbm", 5.0 * k * D * 4),
        # the dweight GEMM that ends in the update of its rows: E and Xs in, W and v in and out;
        # its 2*B*D*k flops need less time at the MFMA peak than these bytes at the HBM peak
        "gemm_dweight_update": ("hbm", float(B) * k * es + float(B) * D * es + 4.0 * k * D * 4),
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    # the first ~20 steps touch rows of W (8.4 GB at the headline workload) for the first time and run
    # ~4 % slower than the steady state
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="headline")
    ap.add_argument("--r", type=float, default=None, help="override the sampling ratio")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fused", action="store_true",
                    help="make `value` the pfc_sample + pfc_forward_backward_update sequence (one "
                         "call for forward/backward and update) instead of the three calls the "
                         "metric names; both sequences are timed and reported either way")
    args = ap.parse_args()
    args.two_calls = not args.fused
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2203_15565_amd import binding, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    wl = workloads.CONFIGS[args.workload]
    if args.r is not None:
        wl = wl.with_(r=args.r)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, Wm = args.steps, args.warmup
    nsteps = K + Wm

    # ---- inputs, resident in HBM before anything is timed --------------------------------
    Wd = torch.empty((wl.N, wl.D), dtype=torch.float32, device=dev)
    for row0, chunk in workloads.weight_chunks(wl):
        Wd[row0:row0 + chunk.shape[0]].copy_(torch.from_numpy(chunk))
    vd = torch.zeros_like(Wd)
    feats = [torch.from_numpy(workloads.make_features(wl, t)).to(dev) for t in range(nsteps)]
    labels_np = [workloads.make_labels(wl, t) for t in range(nsteps)]
    labels = [torch.from_numpy(l).to(dev) for l in labels_np]

    ctx = binding.Context(wl.N, wl.D, wl.B, wl.r, wl.precision)
    cap = binding.pfc_num_sampled(wl.N, wl.B, wl.r)
    idx = torch.zeros(cap, dtype=torch.int32, device=dev)
    yl = torch.zeros(wl.B, dtype=torch.int32, device=dev)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    dX = torch.zeros((wl.B, wl.D), dtype=torch.float32, device=dev)
    dW = torch.zeros((cap, wl.D), dtype=torch.float32, device=dev)

    # One plain element-wise pass of known size (reads and writes k*D*4 bytes), untimed: it is the
    # reference that scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run.
    torch.mul(dW, 1.0, out=dW)

    def step(t: int, two_calls: bool = args.two_calls) -> int:
        k = ctx.pfc_sample(labels[t], wl.r, wl.seed, t, idx, yl)
        if two_calls:
            ctx.pfc_forward_backward(feats[t], Wd, idx, k, yl, wl.s, wl.m, loss, dX, dW)
            ctx.pfc_update(Wd, vd, idx, k, dW, wl.lr, wl.mu)
        else:   # same results; the center gradient stays inside the library
            ctx.pfc_forward_backward_update(feats[t], Wd, vd, idx, k, yl, wl.s, wl.m, wl.lr, wl.mu,
                                            loss, dX)
        return k

    # ---- cpu baseline: the oracle, one whole step on the same inputs (state before any step) --
    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import pfc_oracle as O
        t0 = time.perf_counter()
        oidx, oyl, ok = O.sample(labels_np[0], wl.N, wl.r, wl.seed, 0)
        t_sample = time.perf_counter() - t0
        sel = torch.from_numpy(oidx.astype(np.int64)).to(dev)
        W_S = Wd[sel].cpu().numpy()
        v_S = np.zeros_like(W_S, dtype=np.float64)
        X0 = feats[0].cpu().numpy()
        t0 = time.perf_counter()
        fb = O.forward_backward(X0, W_S, oyl, wl.s, wl.m)
        W_S64 = W_S.astype(np.float64)
        O.update(W_S64, v_S, np.arange(ok), fb["dW"], wl.lr, wl.mu)
        t_rest = time.perf_counter() - t0
        t_oracle = t_sample + t_rest
        try:
            import threadpoolctl
            cores = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        cpu_baseline = {
            "value": wl.B / t_oracle, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": "1 whole step of the %s workload (B=%d, k=%d) in NumPy fp64: sampling %.2f s, "
                      "loss+gradients+update %.2f s" % (wl.name, wl.B, ok, t_sample, t_rest),
            "oracle_loss": fb["loss"],
        }
        del fb, W_S, W_S64, v_S

    # ---- warm-up, then the timed region ---------------------------------------------------
    k = 0
    for t in range(Wm):
        k = step(t)
    torch.cuda.synchronize()
    if ctx.pfc_check() != binding.PFC_OK:
        print("bench.py: device reported an out-of-range label", file=sys.stderr)
        return 1
    first_loss = None
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(Wm, nsteps):
        k = step(t)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / K * 1e3
    value = wl.B * K / elapsed

    # ---- the other call sequence over the same number of steps, for the record ----
    other = not args.two_calls
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(Wm, nsteps):
        step(t, other)
    torch.cuda.synchronize()
    other_elapsed = time.perf_counter() - t0

    # ---- per-call durations: an event pair around every ABI call (the library's stream is torch's
    # current stream, so torch events see it), averaged over the same steps ----
    def timed(fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        r = fn()
        e1.record()
        return r, (e0, e1)

    call_ev: dict = {}
    reps = min(K, 10)
    for t in range(reps):
        tt = Wm + t
        kk, ev = timed(lambda: ctx.pfc_sample(labels[tt], wl.r, wl.seed, tt, idx, yl))
        call_ev.setdefault("pfc_sample", []).append(ev)
        _, ev = timed(lambda: ctx.pfc_forward_backward(feats[tt], Wd, idx, kk, yl, wl.s, wl.m, loss,
                                                       dX, dW))
        call_ev.setdefault("pfc_forward_backward", []).append(ev)
        _, ev = timed(lambda: ctx.pfc_update(Wd, vd, idx, kk, dW, wl.lr, wl.mu))
        call_ev.setdefault("pfc_update", []).append(ev)
        ctx.pfc_sample(labels[tt], wl.r, wl.seed, tt, idx, yl)
        _, ev = timed(lambda: ctx.pfc_forward_backward_update(feats[tt], Wd, vd, idx, kk, yl, wl.s,
                                                              wl.m, wl.lr, wl.mu, loss, dX))
        call_ev.setdefault("pfc_forward_backward_update", []).append(ev)
    torch.cuda.synchronize()
    calls_ms = {n: round(float(np.mean([a.elapsed_time(b) for a, b in evs])), 5)
                for n, evs in call_ev.items()}

    # ---- per-kernel durations: same steps again with an event pair around every kernel, for both
    # call sequences (the timed one last, so that a kernel both use is reported from it) ----
    ctx.pfc_set_timing(True)
    acc: dict = {}
    acc_other: dict = {}
    for which, dst in ((other, acc_other), (args.two_calls, acc)):
        for t in range(reps):
            step(Wm + t, which)
            for name, ms in ctx.pfc_get_timing().items():
                dst.setdefault(name, []).append(ms)
        ctx.pfc_set_timing(True)     # forget the launches of this sequence
    ctx.pfc_set_timing(False)
    kern_ms = {n: float(np.mean(v)) for n, v in acc.items()}
    other_only_ms = {n: float(np.mean(v)) for n, v in acc_other.items() if n not in kern_ms}
    work = algorithmic_work(wl.B, wl.D, k, wl.precision)
    peak_mfma = PEAK_BF16_TFLOPS if wl.precision == 1 else PEAK_FP32_MFMA_TFLOPS
    kernels = {}
    for name, ms in sorted(list(kern_ms.items()) + list(other_only_ms.items()), key=lambda kv: -kv[1]):
        ent = {"ms": round(ms, 5)}
        if name in other_only_ms:
            ent["sequence"] = "other"      # launched only by the call sequence that is not `value`
        if name in work:
            bound, amount = work[name]
            if bound == "mfma":
                ach = amount / (ms * 1e-3) / 1e12
                ent.update(bound="mfma", achieved=round(ach, 2), peak=peak_mfma, unit="TFLOP/s",
                           frac=round(ach / peak_mfma, 4),
                           mfma_busy_frac=MEASURED_MFMA_BUSY.get((wl.name, wl.r, name)))
            else:
                ach = amount / (ms * 1e-3) / 1e9
                ent.update(bound="hbm", achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                           frac=round(ach / PEAK_HBM_GBS, 4),
                           traffic=MEASURED_TRAFFIC_BYTES.get((wl.name, wl.r, name)))
                if name == "gemm_dweight_update":
                    ent["mfma_busy_frac"] = MEASURED_MFMA_BUSY.get((wl.name, wl.r, name))
        kernels[name] = ent
    # the sampler: integer work only (five sweeps of one Philox4x32-10 block per four classes, about
    # 70 integer operations each), so its yardstick is the integer ALU rate, 256 CUs x 64 lanes x
    # 2.4 GHz = 39.3 Tops/s; in practice it is bound by its six dependent launches
    samp_ms = sum(ms for n, ms in kern_ms.items() if n.startswith("sample_"))
    samp_ops = 5.0 * (wl.N / 4.0) * 70.0
    sampler = {"ms": round(samp_ms, 5), "launches": sum(1 for n in kern_ms if n.startswith("sample_")),
               "bound": "alu", "achieved": round(samp_ops / (samp_ms * 1e-3) / 1e12, 3), "peak": 39.3,
               "unit": "Tops/s", "frac": round(samp_ops / (samp_ms * 1e-3) / 1e12 / 39.3, 4)}
    # for comparison, a select that stored one 4-byte score per class and read it once more would
    # move N*4*2 + N + k*4 bytes: that much time at the HBM peak
    stored = wl.N * 4 * 2 + wl.N + k * 4
    sampler["stored_scores_bytes"] = int(stored)
    sampler["stored_scores_ms_at_hbm_peak"] = round(stored / (PEAK_HBM_GBS * 1e9) * 1e3, 5)
    dominant = max((n for n in kern_ms if n in work), key=lambda n: kern_ms[n])
    roofline = {"kernel": dominant}
    roofline.update({f: kernels[dominant][f] for f in ("bound", "achieved", "peak", "unit", "frac")})
    roofline["ms"] = kernels[dominant]["ms"]
    roofline["traffic"] = MEASURED_TRAFFIC_BYTES.get((wl.name, wl.r, dominant))

    # what this GPU sustains on a plain stream copy (k*D*4 bytes each way) and a bare MFMA loop
    scratch = torch.empty_like(dW)
    measured = {
        "stream_copy_GBps": round(binding.pfc_probe_stream_copy(dW, scratch, 10), 1),
        "mfma_bf16_TFLOPps": round(binding.pfc_probe_mfma_bf16(loss, 5), 1),
    }
    del scratch
    # the vendor GEMM on its best shape (square 8192^3, bf16), as a second yardstick for the MFMA side
    try:
        n = 8192
        A = torch.randn(n, n, device=dev, dtype=torch.bfloat16)
        Bm = torch.randn(n, n, device=dev, dtype=torch.bfloat16)
        C = torch.empty(n, n, device=dev, dtype=torch.bfloat16)
        for _ in range(3):
            torch.matmul(A, Bm, out=C)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            torch.matmul(A, Bm, out=C)
        e1.record()
        torch.cuda.synchronize()
        measured["vendor_gemm_8192_bf16_TFLOPps"] = round(2.0 * n ** 3 * 10 / e0.elapsed_time(e1) / 1e9, 1)
        del A, Bm, C
    except Exception:   # the yardstick is optional
        measured["vendor_gemm_8192_bf16_TFLOPps"] = None
    ref = measured["stream_copy_GBps"] if roofline["bound"] == "hbm" else measured["mfma_bf16_TFLOPps"]
    roofline["frac_of_measured_peak"] = round(roofline["achieved"] / ref, 4)

    out = {
        "metric": "PFC fwd+bwd+update samples/s",
        "value": round(value, 1),
        "unit": "samples/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": Wm,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if wl.precision == 1 else "f32",
        "data": "synthetic",
        "config": {"workload": "%s: B=%d D=%d N=%d r=%g k=%d, Zipf(%.1f) labels, s=%g m=%g, "
                               "SGD lr=%g mu=%g" % (wl.name, wl.B, wl.D, wl.N, wl.r, k,
                                                    wl.zipf_alpha, wl.s, wl.m, wl.lr, wl.mu),
                   "B": wl.B, "D": wl.D, "N": wl.N, "r": wl.r, "k": k,
                   "calls": "pfc_sample + pfc_forward_backward + pfc_update" if args.two_calls
                   else "pfc_sample + pfc_forward_backward_update"},
        # both sequences side by side, whichever one `value` is
        "value_three_calls": round(value if args.two_calls else wl.B * K / other_elapsed, 1),
        "value_fused_call": round(wl.B * K / other_elapsed if args.two_calls else value, 1),
        "calls_ms": calls_ms,
        "other_call_sequence": {
            "calls": "pfc_sample + pfc_forward_backward + pfc_update" if other
            else "pfc_sample + pfc_forward_backward_update",
            "ms_per_step": round(other_elapsed / K * 1e3, 4),
            "value": round(wl.B * K / other_elapsed, 1)},
        # the paper times whole training jobs on other hardware: context, not a baseline
        "paper_context": "Tab. 6: PFC-0.1 at 2M identities, 3552 samples/s end to end on 8 x V100 "
                         "(fp16 AMP, ResNet100 backbone included)" if wl.name == "headline" else None,
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "measured_peaks": measured,
        "sampler": sampler,
        "kernels": kernels,
        "kernel_sum_ms": round(sum(kern_ms.values()), 4),
        "final_loss": float(loss.item()),
    }
    print(json.dumps(out))
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
