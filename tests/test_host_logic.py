"""CPU tests of the host-side logic around the library: the input generators, the benchmark's
bookkeeping and its refusal of more than one GPU."""
from __future__ import annotations

import os
import subprocess
import sys

import numpy as np
import pytest

from paper_2203_15565_amd import binding, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode == 2
    assert "ONE GPU" in p.stderr and p.stdout.strip() == ""


def test_algorithmic_work_of_the_headline_step():
    sys.path.insert(0, ROOT)
    import bench
    B, D, k = 1024, 512, 205_991
    w = bench.algorithmic_work(B, D, k, 1)
    for name in ("gemm_logits", "gemm_dweight", "gemm_dfeatures"):
        assert w[name] == ("mfma", 2.0 * B * D * k)
    assert w["update"] == ("hbm", 5.0 * k * D * 4)
    assert w["gather_normalize_w"] == ("hbm", k * D * 6 + 4.0 * k)
    # fused kernel: E and Xs (bf16) in, W and v (fp32) in and out
    assert w["gemm_dweight_update"] == ("hbm", B * k * 2.0 + B * D * 2.0 + 4.0 * k * D * 4)


def test_workload_table_matches_the_benchmark_configurations():
    c = workloads.CONFIGS
    assert (c["tiny"].B, c["tiny"].N, c["tiny"].precision) == (128, 10_000, 0)
    assert (c["medium"].B, c["medium"].N) == (512, 93_431)
    assert (c["large"].B, c["large"].N) == (1024, 360_232)
    assert (c["headline"].B, c["headline"].N, c["headline"].r) == (1024, 2_059_906, 0.1)
    assert (c["extreme"].B, c["extreme"].N) == (2048, 10_000_000)   # 10M classes as in Tab. 6
    assert all(w.D == 512 and w.s == 64.0 and w.m == 0.5 for w in c.values())
    for w in c.values():
        assert binding.pfc_num_sampled(w.N, w.B, w.r) >= w.B


def test_generators_are_reproducible_and_in_range():
    wl = workloads.CONFIGS["medium"]
    a, b = workloads.make_labels(wl, 3), workloads.make_labels(wl, 3)
    assert a.dtype == np.int64 and a.shape == (wl.B,) and np.array_equal(a, b)
    assert a.min() >= 0 and a.max() < wl.N
    assert not np.array_equal(a, workloads.make_labels(wl, 4))
    X = workloads.make_features(wl, 0)
    assert X.dtype == np.float32 and X.shape == (wl.B, wl.D)
    assert np.array_equal(X, workloads.make_features(wl, 0))
    assert abs(float(X.mean())) < 0.02 and abs(float(X.std()) - 1.0) < 0.02


def test_random_streams_of_the_generators_never_coincide():
    """Features, labels, centers and the permutation draw from separate streams for every config
    and step: no batch of features is a multiple of rows of the center matrix (which would make
    cosines of exactly 1 and the projected center gradient a pure rounding residue)."""
    heads = {}
    for wl in workloads.CONFIGS.values():
        small = wl.with_(B=2, N=min(wl.N, 64))
        for row0, chunk in workloads.weight_chunks(small):
            heads[("W", wl.name)] = tuple(np.round(chunk[0, :6] * 100, 4))
        for t in range(12):
            heads[("X", wl.name, t)] = tuple(np.round(workloads.make_features(small, t)[0, :6], 4))
    assert len(set(heads.values())) == len(heads)


def test_zipf_labels_are_long_tailed():
    wl = workloads.CONFIGS["large"]
    lab = np.concatenate([workloads.make_labels(wl, t) for t in range(20)])
    _, counts = np.unique(lab, return_counts=True)
    # a few head classes own a large share of the samples, most classes appear once
    assert counts.max() > 50 * np.median(counts)
    assert np.mean(counts == 1) > 0.5
    # and the head classes are spread over the id range by the seeded permutation
    top = np.argsort(np.bincount(lab, minlength=wl.N))[-8:]
    assert top.max() - top.min() > wl.N // 4


def test_weight_chunks_tile_the_matrix():
    wl = workloads.CONFIGS["tiny"]
    W = workloads.make_weight(wl)
    assert W.shape == (wl.N, wl.D) and W.dtype == np.float32
    rows = 0
    for row0, chunk in workloads.weight_chunks(wl, rows_per_chunk=4096):
        assert row0 == rows
        rows += chunk.shape[0]
    assert rows == wl.N
    assert abs(float(W.std()) - 0.01) < 2e-4     # N(0, 0.01^2)


def test_fused_entry_point_rejects_a_null_context():
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("libpfc.so not built (run python -m paper_2203_15565_amd.build)")
    lib = binding.load()
    rc = lib.pfc_forward_backward_update(None, None, None, None, None, 1, None, 1, 64.0, 0.5, 0,
                                         2.0, 0.1, 0.9, None, None, None)
    assert rc == binding.PFC_EINVAL
