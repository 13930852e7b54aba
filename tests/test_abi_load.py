"""The C-ABI library loads and exports every symbol that include/pfc.h declares (no GPU needed),
and the host-side argument checks that never touch the device behave as documented."""
import ctypes
import math
import os
import re

import pytest

from paper_2203_15565_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols(header="pfc.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pfc_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("libpfc.so not built (run python -m paper_2203_15565_amd.build)")
    lib = ctypes.CDLL(binding.LIB_PATH)
    declared = _declared_symbols()
    assert len(declared) >= 10
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == declared


def test_probe_header_symbols_are_exported():
    if not os.path.exists(binding.PROBE_LIB_PATH):
        pytest.skip("libpfc_probe.so not built (run python -m paper_2203_15565_amd.build)")
    lib = ctypes.CDLL(binding.PROBE_LIB_PATH)
    declared = _declared_symbols("pfc_probe.h")
    assert declared == sorted(binding.PROBE_EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    # and the product library no longer carries them
    if os.path.exists(binding.LIB_PATH):
        prod = ctypes.CDLL(binding.LIB_PATH)
        assert not any(hasattr(prod, name) for name in declared)


def test_num_sampled_host_function():
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("libpfc.so not built")
    f = binding.pfc_num_sampled
    assert f(10_000, 128, 0.1) == 1000
    assert f(93_431, 512, 0.1) == 9344
    assert f(360_232, 1024, 0.1) == 36024
    assert f(2_059_906, 1024, 0.05) == 102_996
    assert f(2_059_906, 1024, 0.1) == 205_991
    assert f(2_059_906, 1024, 0.2) == 411_982
    assert f(2_059_906, 1024, 0.4) == 823_963
    assert f(10_000_000, 2048, 0.05) == 500_000
    assert f(1000, 64, 0.001) == 64          # capacity bound max(B, ceil(rN))
    assert f(100, 64, 1.0) == 100
    assert f(0, 64, 0.5) == -1 and f(10, 0, 0.5) == -1 and f(10, 4, 0.0) == -1
    assert f(10, 4, 1.5) == -1 and f(1 << 31, 4, 0.5) == -1


def test_strerror():
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("libpfc.so not built")
    lib = binding.load()
    assert lib.pfc_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4):
        assert len(lib.pfc_strerror(code)) > 0


def test_null_context_is_einval():
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("libpfc.so not built")
    lib = binding.load()
    k = ctypes.c_int64(0)
    assert lib.pfc_sample(None, None, 1, 0.5, 0, 0, None, None, ctypes.byref(k)) == binding.PFC_EINVAL
    assert lib.pfc_forward_backward(None, None, None, None, 1, None, 1, 64.0, 0.5, None, None,
                                    None) == binding.PFC_EINVAL
    assert lib.pfc_update(None, None, None, None, 1, None, 0.1, 0.9) == binding.PFC_EINVAL
    assert lib.pfc_check(None) == binding.PFC_EINVAL
    assert lib.pfc_destroy(None) == binding.PFC_EINVAL


def test_create_rejects_what_the_header_rules_out():
    """Argument checks of pfc_create that return before any device call."""
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("libpfc.so not built")
    lib = binding.load()
    h = ctypes.c_void_p()
    bad = [
        (1000, 300, 64, 0.1, 1),              # D not a multiple of 64
        (1000, 32, 64, 0.1, 1),               # D below 64
        (1000, 1280, 64, 0.1, 1),             # D above 1024
        (0, 512, 64, 0.1, 1), (1 << 31, 512, 64, 0.1, 1),
        (1000, 512, 0, 0.1, 1), (1000, 512, 64, 0.0, 1), (1000, 512, 64, 1.5, 1),
        (1000, 512, 64, 0.1, 2),              # unknown precision
        ((1 << 31) - 1, 512, 1024, 1.0, 1),   # 2^31 sampled classes: beyond the 32-bit staging offsets
        (1 << 25, 512, 1024, 1.0, 0),         # 2^25 sampled classes with fp32 operands: likewise
    ]
    for N, D, B, r, prec in bad:
        rc = lib.pfc_create(ctypes.byref(h), N, D, B, r, prec, None)
        assert rc == binding.PFC_EINVAL and not h.value, (N, D, B, r, prec, rc)
    assert lib.pfc_create(None, 1000, 512, 64, 0.1, 1, None) == binding.PFC_EINVAL


def test_library_is_not_older_than_its_sources():
    """Guards against running GPU tests on a stale build: rebuild after touching csrc/."""
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("libpfc.so not built")
    lib_m = os.path.getmtime(binding.LIB_PATH)
    csrc = os.path.join(ROOT, "paper_2203_15565_amd", "csrc")
    srcs = [os.path.join(csrc, f) for f in os.listdir(csrc)] + [os.path.join(ROOT, "include", "pfc.h")]
    newest = max(os.path.getmtime(p) for p in srcs)
    assert lib_m >= newest, "libpfc.so is older than its sources: run python -m paper_2203_15565_amd.build"
