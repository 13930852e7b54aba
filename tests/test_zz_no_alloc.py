"""pfc_sample_noalloc (the entry point that allocates nothing: its scratch is a static device
array of the library) against pfc_sample, through the C ABI: bit-identical ids and local labels on
two calls in a row, the second with a smaller input, so that whatever the first call left in the
shared array would show."""
import sys

import numpy as np
import pytest

from paper_2203_15565_amd import binding, workloads

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _both(N, B, r, labels_np, seed, step):
    import torch
    cap = binding.pfc_num_sampled(N, B, r)
    labels = torch.from_numpy(np.ascontiguousarray(labels_np, dtype=np.int64)).cuda()
    out = []
    for which in ("ctx", "noalloc"):
        idx = torch.full((cap,), -7, dtype=torch.int32, device="cuda")
        yl = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        if which == "ctx":
            ctx = binding.Context(N, 256, B, r, binding.PRECISION_BF16)
            k = ctx.pfc_sample(labels, r, seed, step, idx, yl)
            torch.cuda.synchronize()
            assert ctx.pfc_check() == binding.PFC_OK
            ctx.close()
        else:
            k = binding.pfc_sample_noalloc(labels, N, r, seed, step, idx, yl)
            torch.cuda.synchronize()
        out.append((k, idx.cpu().numpy(), yl.cpu().numpy()))
    (ka, ia, ya), (kb, ib, yb) = out
    assert ka == kb
    assert np.array_equal(ia, ib)          # includes the untouched tail past k
    assert np.array_equal(ya, yb)
    assert np.array_equal(ib[yb], labels_np)
    return kb


def test_noalloc_sample_matches_pfc_sample_twice_in_a_row():
    wl = workloads.CONFIGS["headline"]
    _say("noalloc: headline sized call")
    k1 = _both(wl.N, wl.B, wl.r, workloads.make_labels(wl, 0), wl.seed, 0)
    assert k1 == 205_991
    # second call: fewer classes, smaller batch, ragged against every block size, other step
    N2, B2, r2 = 70_001, 300, 0.05
    labels2 = np.random.default_rng(8).integers(0, N2, size=B2)
    _say("noalloc: smaller call")
    k2 = _both(N2, B2, r2, labels2, 11, 3)
    assert k2 == 3501
    # and a third, larger again, with duplicates and r = 1
    N3, B3 = 5000, 64
    labels3 = np.full(B3, 4999)
    labels3[:7] = [0, 1, 2, 3, 31, 32, 2048]
    _say("noalloc: r = 1")
    assert _both(N3, B3, 1.0, labels3, 1, 2) == N3


def test_noalloc_sample_rejects_what_it_cannot_do():
    import torch
    labels = torch.zeros(64, dtype=torch.int64, device="cuda")
    idx = torch.zeros(1 << 12, dtype=torch.int32, device="cuda")
    yl = torch.zeros(64, dtype=torch.int32, device="cuda")
    for N, r in (((1 << 24) + 1, 0.0001),      # beyond the static scratch
                 (10_000, 0.001),              # ceil(r N) = 10 < B: k would depend on the labels
                 (10_000, 0.0), (10_000, 1.5), (0, 0.5)):
        with pytest.raises(binding.PfcError) as e:
            binding.pfc_sample_noalloc(labels, N, r, 0, 0, idx, yl)
        assert e.value.code == binding.PFC_EINVAL
    torch.cuda.synchronize()
