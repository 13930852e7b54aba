"""ctypes binding of libpfc.so: argument marshalling only.

Every function mirrors one entry point of include/pfc.h and passes raw device pointers of torch
tensors (torch is used for device memory and streams, nothing else).  There is no CPU fallback:
if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpfc.so")
PROBE_LIB_PATH = os.path.join(_HERE, "libpfc_probe.so")

PFC_OK = 0
PFC_EINVAL = -1
PFC_ELABEL = -2
PFC_EHIP = -3
PFC_ENOMEM = -4
PRECISION_FP32 = 0
PRECISION_BF16 = 1
MARGIN_ARCFACE = 0
MARGIN_COSFACE = 1

EXPORTS = [
    "pfc_create", "pfc_destroy", "pfc_num_sampled", "pfc_sample", "pfc_sample_masked",
    "pfc_sample_noalloc",
    "pfc_forward_backward", "pfc_forward_backward_ex", "pfc_forward_backward_update", "pfc_update", "pfc_check", "pfc_set_timing", "pfc_get_timing",
    "pfc_strerror", "pfc_last_hip_error",
]
PROBE_EXPORTS = ["pfc_probe_stream_copy", "pfc_probe_mfma_bf16"]

_lib: Optional[ctypes.CDLL] = None


class PfcError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        lib = load()
        msg = lib.pfc_strerror(code).decode()
        if code == PFC_EHIP:
            msg += " (" + lib.pfc_last_hip_error().decode() + ")"
        super().__init__("%s failed: %s [%d]" % (where, msg, code))


def load() -> ctypes.CDLL:
    """Load libpfc.so (built in-tree by paper_2203_15565_amd.build); raise if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            LIB_PATH + " is missing: run `python -m paper_2203_15565_amd.build` first "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    c = ctypes
    vp, i32, i64, u32, u64, f32, f64 = (c.c_void_p, c.c_int32, c.c_int64, c.c_uint32, c.c_uint64,
                                        c.c_float, c.c_double)
    lib.pfc_create.argtypes = [c.POINTER(vp), i64, i32, i32, f64, i32, vp]
    lib.pfc_create.restype = c.c_int
    lib.pfc_destroy.argtypes = [vp]
    lib.pfc_destroy.restype = c.c_int
    lib.pfc_num_sampled.argtypes = [i64, i32, f64]
    lib.pfc_num_sampled.restype = i64
    lib.pfc_sample.argtypes = [vp, vp, i32, f64, u64, u64, vp, vp, c.POINTER(i64)]
    lib.pfc_sample.restype = c.c_int
    lib.pfc_sample_masked.argtypes = [vp, vp, i32, f64, u64, u64, u32, vp, vp, c.POINTER(i64)]
    lib.pfc_sample_masked.restype = c.c_int
    lib.pfc_sample_noalloc.argtypes = [vp, i32, i64, f64, u64, u64, vp, vp, c.POINTER(i64), vp]
    lib.pfc_sample_noalloc.restype = c.c_int
    lib.pfc_forward_backward.argtypes = [vp, vp, vp, vp, i64, vp, i32, f32, f32, vp, vp, vp]
    lib.pfc_forward_backward.restype = c.c_int
    lib.pfc_forward_backward_ex.argtypes = [vp, vp, vp, vp, i64, vp, i32, f32, f32, i32, f32, vp, vp,
                                            vp, vp]
    lib.pfc_forward_backward_ex.restype = c.c_int
    lib.pfc_forward_backward_update.argtypes = [vp, vp, vp, vp, vp, i64, vp, i32, f32, f32, i32, f32,
                                                f32, f32, vp, vp, vp]
    lib.pfc_forward_backward_update.restype = c.c_int
    lib.pfc_update.argtypes = [vp, vp, vp, vp, i64, vp, f32, f32]
    lib.pfc_update.restype = c.c_int
    lib.pfc_check.argtypes = [vp]
    lib.pfc_check.restype = c.c_int
    lib.pfc_set_timing.argtypes = [vp, i32]
    lib.pfc_set_timing.restype = c.c_int
    lib.pfc_get_timing.argtypes = [vp, c.POINTER(c.c_char_p), c.POINTER(f32), i32]
    lib.pfc_get_timing.restype = c.c_int
    lib.pfc_strerror.argtypes = [c.c_int]
    lib.pfc_strerror.restype = c.c_char_p
    lib.pfc_last_hip_error.argtypes = []
    lib.pfc_last_hip_error.restype = c.c_char_p
    _lib = lib
    return lib


_probe_lib: Optional[ctypes.CDLL] = None


def load_probe() -> ctypes.CDLL:
    """Load libpfc_probe.so (the benchmark's calibration probes); raise if it is missing."""
    global _probe_lib
    if _probe_lib is None:
        if not os.path.exists(PROBE_LIB_PATH):
            raise FileNotFoundError(PROBE_LIB_PATH + " is missing: run "
                                    "`python -m paper_2203_15565_amd.build` first")
        lib = ctypes.CDLL(PROBE_LIB_PATH)
        c = ctypes
        lib.pfc_probe_stream_copy.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64,
                                              c.c_int32, c.POINTER(c.c_double)]
        lib.pfc_probe_stream_copy.restype = c.c_int
        lib.pfc_probe_mfma_bf16.argtypes = [c.c_void_p, c.c_void_p, c.c_int32,
                                            c.POINTER(c.c_double)]
        lib.pfc_probe_mfma_bf16.restype = c.c_int
        _probe_lib = lib
    return _probe_lib


def _current_stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def pfc_probe_stream_copy(src, dst, reps: int = 10) -> float:
    """GB/s (read + write) of a plain copy of src into dst (same-size device tensors)."""
    out = ctypes.c_double(0.0)
    nbytes = src.numel() * src.element_size()
    rc = load_probe().pfc_probe_stream_copy(ctypes.c_void_p(_current_stream()), _ptr(src),
                                            _ptr(dst), nbytes, reps, ctypes.byref(out))
    if rc != PFC_OK:
        raise RuntimeError("pfc_probe_stream_copy failed [%d]" % rc)
    return float(out.value)


def pfc_probe_mfma_bf16(sink, reps: int = 5) -> float:
    """TFLOP/s of a bare bf16 MFMA issue loop (sink: any device float tensor)."""
    out = ctypes.c_double(0.0)
    rc = load_probe().pfc_probe_mfma_bf16(ctypes.c_void_p(_current_stream()), _ptr(sink), reps,
                                          ctypes.byref(out))
    if rc != PFC_OK:
        raise RuntimeError("pfc_probe_mfma_bf16 failed [%d]" % rc)
    return float(out.value)


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def pfc_num_sampled(N: int, B: int, r: float) -> int:
    return int(load().pfc_num_sampled(N, B, float(r)))


def pfc_sample_noalloc(labels, N: int, r: float, seed: int, step: int, idx_out, labels_local_out,
                       stream: Optional[int] = None) -> int:
    """pfc_sample without a context and without any allocation (static device scratch); returns k."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    k = ctypes.c_int64(0)
    rc = load().pfc_sample_noalloc(_ptr(labels), labels.numel(), N, float(r), seed, step,
                                   _ptr(idx_out), _ptr(labels_local_out), ctypes.byref(k),
                                   ctypes.c_void_p(stream))
    if rc != PFC_OK:
        raise PfcError(rc, "pfc_sample_noalloc")
    return int(k.value)


class Context:
    """Owner of one pfc_ctx (scratch for problems up to N, D, B_max, r_max on one stream)."""

    def __init__(self, N: int, D: int, B_max: int, r_max: float, precision: int,
                 stream: Optional[int] = None):
        lib = load()
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        self._h = ctypes.c_void_p()
        rc = lib.pfc_create(ctypes.byref(self._h), N, D, B_max, float(r_max), precision,
                            ctypes.c_void_p(stream))
        if rc != PFC_OK:
            self._h = ctypes.c_void_p()
            raise PfcError(rc, "pfc_create")
        self.N, self.D, self.B_max, self.r_max, self.precision = N, D, B_max, r_max, precision

    def close(self) -> None:
        if self._h:
            load().pfc_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- entry points ---------------------------------------------------------------------
    def pfc_sample(self, labels, r: float, seed: int, step: int, idx_out, labels_local_out,
                   score_mask: Optional[int] = None) -> int:
        """labels: int64[B] cuda; idx_out: int32[>= pfc_num_sampled]; returns exact k."""
        k = ctypes.c_int64(0)
        B = labels.numel()
        lib = load()
        if score_mask is None:
            rc = lib.pfc_sample(self._h, _ptr(labels), B, float(r), seed, step, _ptr(idx_out),
                                _ptr(labels_local_out), ctypes.byref(k))
        else:
            rc = lib.pfc_sample_masked(self._h, _ptr(labels), B, float(r), seed, step, score_mask,
                                       _ptr(idx_out), _ptr(labels_local_out), ctypes.byref(k))
        if rc != PFC_OK:
            raise PfcError(rc, "pfc_sample")
        return int(k.value)

    def pfc_forward_backward(self, features, weight, idx, k: int, labels_local, s: float,
                             m: float, loss_out, dfeatures_out, dweight_out) -> None:
        rc = load().pfc_forward_backward(self._h, _ptr(features), _ptr(weight), _ptr(idx), k,
                                         _ptr(labels_local), features.shape[0], s, m,
                                         _ptr(loss_out), _ptr(dfeatures_out), _ptr(dweight_out))
        if rc != PFC_OK:
            raise PfcError(rc, "pfc_forward_backward")

    def pfc_forward_backward_ex(self, features, weight, idx, k: int, labels_local, s: float,
                                m: float, margin_type: int, filter_threshold: float, loss_out,
                                dfeatures_out, dweight_out, stats_out=None) -> None:
        rc = load().pfc_forward_backward_ex(self._h, _ptr(features), _ptr(weight), _ptr(idx), k,
                                            _ptr(labels_local), features.shape[0], s, m,
                                            margin_type, filter_threshold, _ptr(loss_out),
                                            _ptr(dfeatures_out), _ptr(dweight_out),
                                            _ptr(stats_out))
        if rc != PFC_OK:
            raise PfcError(rc, "pfc_forward_backward_ex")

    def pfc_forward_backward_update(self, features, weight, momentum, idx, k: int, labels_local,
                                    s: float, m: float, lr: float, mu: float, loss_out,
                                    dfeatures_out, margin_type: int = MARGIN_ARCFACE,
                                    filter_threshold: float = 2.0, stats_out=None) -> None:
        rc = load().pfc_forward_backward_update(self._h, _ptr(features), _ptr(weight),
                                                _ptr(momentum), _ptr(idx), k, _ptr(labels_local),
                                                features.shape[0], s, m, margin_type,
                                                filter_threshold, lr, mu, _ptr(loss_out),
                                                _ptr(dfeatures_out), _ptr(stats_out))
        if rc != PFC_OK:
            raise PfcError(rc, "pfc_forward_backward_update")

    def pfc_update(self, weight, momentum, idx, k: int, dweight, lr: float, mu: float) -> None:
        rc = load().pfc_update(self._h, _ptr(weight), _ptr(momentum), _ptr(idx), k, _ptr(dweight),
                               lr, mu)
        if rc != PFC_OK:
            raise PfcError(rc, "pfc_update")

    def pfc_check(self) -> int:
        return int(load().pfc_check(self._h))

    def check(self) -> None:
        rc = self.pfc_check()
        if rc != PFC_OK:
            raise PfcError(rc, "pfc_check")

    def pfc_set_timing(self, enabled: bool) -> None:
        rc = load().pfc_set_timing(self._h, 1 if enabled else 0)
        if rc != PFC_OK:
            raise PfcError(rc, "pfc_set_timing")

    def pfc_get_timing(self) -> dict:
        cap = 64
        names = (ctypes.c_char_p * cap)()
        ms = (ctypes.c_float * cap)()
        n = load().pfc_get_timing(self._h, names, ms, cap)
        if n < 0:
            raise PfcError(n, "pfc_get_timing")
        return {names[i].decode(): float(ms[i]) for i in range(n)}
