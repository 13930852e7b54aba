"""Seeded synthetic inputs for the Partial FC step.

This module holds NO arithmetic of the method: it only draws features, labels and initial
centers with the shapes and distributions of the paper's workloads (arXiv 2203.15565,
Sec. 4.1: WebFace4M / 12M / 42M have 200K / 600K / 2M identities; Tab. 6: "synthetic 10M
identities"; Sec. 3.1, second limitation: identities are long-tailed, 44.57 % of them with
fewer than 10 images).  The same arrays are handed to the HIP path and to the CPU oracle.

Everything is NumPy on the host (PCG64), so a given (config, step) is reproducible on any
machine.  The large center matrices are generated in row chunks to bound host memory.

Every stream of random numbers is seeded with the sequence (stream tag, config id, index): tag 1
features (index = step), 2 labels (index = step), 3 initial centers (index = row chunk), 4 the
class-id permutation.  The tags keep the streams apart whatever the ids are: NumPy pads a seed
sequence with zeros, so plain integer seeds such as 1000*config + step and 3000 + config can name
the same stream (config 3, step 3), which once made a batch of features an exact multiple of the
first rows of the center matrix.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

__all__ = ["Workload", "CONFIGS", "make_features", "make_labels", "weight_chunks",
           "make_weight", "zipf_cdf"]


@dataclass(frozen=True)
class Workload:
    """One named workload.  `precision`: 0 = fp32 GEMM operands, 1 = bf16 GEMM operands."""
    name: str
    cfg_id: int
    B: int
    D: int
    N: int
    r: float
    precision: int
    steps: int
    label_dist: str          # "uniform" or "zipf"
    zipf_alpha: float = 0.0
    s: float = 64.0
    m: float = 0.5
    lr: float = 0.1
    mu: float = 0.9
    seed: int = 0            # sampling seed of the method

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


CONFIGS = {
    "tiny": Workload("tiny", 1, B=128, D=512, N=10_000, r=0.1, precision=0, steps=1,
                     label_dist="uniform"),
    "medium": Workload("medium", 2, B=512, D=512, N=93_431, r=0.1, precision=1, steps=10,
                       label_dist="zipf", zipf_alpha=1.1),
    "large": Workload("large", 3, B=1024, D=512, N=360_232, r=0.1, precision=1, steps=10,
                      label_dist="zipf", zipf_alpha=1.1),
    "headline": Workload("headline", 4, B=1024, D=512, N=2_059_906, r=0.1, precision=1,
                         steps=1, label_dist="zipf", zipf_alpha=1.2),
    "extreme": Workload("extreme", 5, B=2048, D=512, N=10_000_000, r=0.05, precision=1,
                        steps=1, label_dist="zipf", zipf_alpha=1.2),
    # The paper's fastest setting (Sec. 3.3; Tab. 7 caption): no negative outside the batch is
    # drawn (r below B/N, so k = number of distinct labels) and the batch is enlarged to 8K / 16K.
    "ultrafast8k": Workload("ultrafast8k", 6, B=8192, D=512, N=2_059_906, r=1e-9, precision=1,
                            steps=1, label_dist="zipf", zipf_alpha=1.2),
    "ultrafast16k": Workload("ultrafast16k", 7, B=16384, D=512, N=2_059_906, r=1e-9, precision=1,
                             steps=1, label_dist="zipf", zipf_alpha=1.2),
}


_TAG_FEATURES, _TAG_LABELS, _TAG_WEIGHT, _TAG_PERM = 1, 2, 3, 4


def make_features(wl: Workload, step: int) -> np.ndarray:
    """B x D i.i.d. N(0,1) fp32 features, fresh for every step."""
    rng = np.random.default_rng([_TAG_FEATURES, wl.cfg_id, step])
    return rng.standard_normal((wl.B, wl.D), dtype=np.float32)


_zipf_cache: dict = {}


def zipf_cdf(N: int, alpha: float) -> np.ndarray:
    """fp64 CDF of P(rank t) ~ t^-alpha over ranks 1..N."""
    key = (N, alpha)
    if key not in _zipf_cache:
        w = np.arange(1, N + 1, dtype=np.float64) ** (-alpha)
        cdf = np.cumsum(w)
        cdf /= cdf[-1]
        _zipf_cache.clear()
        _zipf_cache[key] = cdf
    return _zipf_cache[key]


_perm_cache: dict = {}


def _class_perm(wl: Workload) -> np.ndarray:
    key = (wl.cfg_id, wl.N)
    if key not in _perm_cache:
        _perm_cache.clear()
        _perm_cache[key] = np.random.default_rng([_TAG_PERM, wl.cfg_id]).permutation(wl.N)
    return _perm_cache[key]


def make_labels(wl: Workload, step: int) -> np.ndarray:
    """int64[B] labels: uniform over the classes, or long-tailed (Zipf over a seeded random
    permutation of the class ids, so that frequent classes are spread over the id range)."""
    rng = np.random.default_rng([_TAG_LABELS, wl.cfg_id, step])
    if wl.label_dist == "uniform":
        return rng.integers(0, wl.N, size=wl.B, dtype=np.int64)
    if wl.label_dist == "zipf":
        cdf = zipf_cdf(wl.N, wl.zipf_alpha)
        rank = np.searchsorted(cdf, rng.random(wl.B), side="left")
        rank = np.minimum(rank, wl.N - 1)
        return _class_perm(wl)[rank].astype(np.int64)
    raise ValueError(wl.label_dist)


def weight_chunks(wl: Workload, rows_per_chunk: int = 1 << 18):
    """Yield (row0, chunk) of the initial center matrix: i.i.d. N(0, 0.01^2) fp32.
    Chunk c is drawn from its own generator, so any chunk can be regenerated alone."""
    row0 = 0
    c = 0
    while row0 < wl.N:
        n = min(rows_per_chunk, wl.N - row0)
        rng = np.random.default_rng([_TAG_WEIGHT, wl.cfg_id, c])
        chunk = rng.standard_normal((n, wl.D), dtype=np.float32)
        chunk *= np.float32(0.01)
        yield row0, chunk
        row0 += n
        c += 1


def make_weight(wl: Workload) -> np.ndarray:
    """Whole N x D fp32 initial center matrix on the host (use weight_chunks for big N)."""
    W = np.empty((wl.N, wl.D), dtype=np.float32)
    for row0, chunk in weight_chunks(wl):
        W[row0:row0 + chunk.shape[0]] = chunk
    return W
