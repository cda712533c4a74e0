"""Thin Python binding of the C ABI in ``include/gravac.h``.

Argument marshalling only: every step of the compression path runs in the HIP
kernels of ``libgravac.so``.  PyTorch supplies device memory and the stream.
There is no CPU fallback: if the library cannot be loaded the import of the
first entry point raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

from . import _build

OK = 0
ERR_INVALID_ARG = -1
ERR_CAPACITY = -2
ERR_WORKSPACE = -3
ERR_HIP = -4
ERR_CAPTURE = -5
ERR_STATIC_LIMIT = -6
STATIC_SCRATCH_BYTES = 4 << 20
MAX_CF = 8
FLAG_FORCE_FALLBACK = 1
FLAG_NO_COMMIT = 2

EXPORTS = (
    "gravac_topk_count", "gravac_workspace_bytes", "gravac_compress", "gravac_compress_profiled", "gravac_randomk_compress", "gravac_threshold_compress", "gravac_recompress", "gravac_commit",
    "gravac_decompress_workspace_bytes", "gravac_decompress_accumulate", "gravac_decompress_accumulate_static",
    "gravac_decompress_update",
    "gravac_read_status", "gravac_strerror",
    "gravac_controller_create", "gravac_controller_destroy", "gravac_controller_candidates",
    "gravac_controller_decide", "gravac_controller_finish_iteration", "gravac_controller_throughput",
    "gravac_controller_iteration",
)

POLICY_EXPONENTIAL = 0
POLICY_GEOMETRIC = 1
SEND_CANDIDATE = 0
SEND_MIN = 1
SEND_DENSE = 2


class ControllerConfig(ctypes.Structure):
    """``gravac_controller_config`` of the C ABI."""
    _fields_ = [("theta_min", ctypes.c_double), ("theta_max", ctypes.c_double), ("epsilon", ctypes.c_double),
                ("omega", ctypes.c_double), ("theta_s", ctypes.c_double), ("alpha", ctypes.c_double),
                ("samples_per_iteration", ctypes.c_double), ("window", ctypes.c_int64),
                ("policy", ctypes.c_int32), ("reserved", ctypes.c_int32)]



class ProfileEvents(ctypes.Structure):
    """``gravac_profile_events`` of the C ABI (``include/gravac_profile.h``): four hipEvent_t handles."""
    _fields_ = [("call_begin", ctypes.c_void_p), ("pass_begin", ctypes.c_void_p), ("pass_end", ctypes.c_void_p),
                ("call_end", ctypes.c_void_p)]


_lib = None


class GravacError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code})")


def library_path() -> str:
    return _build.LIBRARY


def lib() -> ctypes.CDLL:
    """Load ``libgravac.so`` (building it first only if no built library exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIBRARY):
            _build.build_library()
        L = ctypes.CDLL(_build.LIBRARY)
        vp, i64, i32, u32, dbl = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_uint, ctypes.c_double
        L.gravac_topk_count.restype = i64
        L.gravac_topk_count.argtypes = [i64, dbl]
        L.gravac_workspace_bytes.restype = i32
        L.gravac_workspace_bytes.argtypes = [i64, i32, i32, ctypes.POINTER(ctypes.c_size_t)]
        L.gravac_compress.restype = i32
        L.gravac_compress.argtypes = [vp, vp, i64, vp, i32, i32, vp, i32, vp, vp, i64, vp, vp, vp,
                                      ctypes.c_size_t, u32, vp]
        L.gravac_compress_profiled.restype = i32
        L.gravac_compress_profiled.argtypes = [vp, vp, i64, vp, i32, i32, vp, i32, vp, vp, i64, vp, vp, vp,
                                               ctypes.c_size_t, u32, vp, ctypes.POINTER(ProfileEvents)]
        L.gravac_randomk_compress.restype = i32
        L.gravac_randomk_compress.argtypes = [vp, vp, i64, vp, i32, i32, ctypes.c_uint64, vp, i32, vp, vp, i64, vp, vp, vp,
                                              ctypes.c_size_t, u32, vp]
        L.gravac_threshold_compress.restype = i32
        L.gravac_threshold_compress.argtypes = [vp, vp, i64, ctypes.c_float, vp, vp, i64, vp, vp, vp, ctypes.c_size_t, vp]
        L.gravac_recompress.restype = i32
        L.gravac_recompress.argtypes = [vp, vp, i64, dbl, vp, i32, vp, i64, vp, vp, i64, vp, vp, vp,
                                        ctypes.c_size_t, u32, vp]
        L.gravac_commit.restype = i32
        L.gravac_commit.argtypes = [vp, i64, vp, i64, vp]
        L.gravac_decompress_accumulate.restype = i32
        L.gravac_decompress_accumulate.argtypes = [vp, vp, vp, i32, i64, vp, vp, ctypes.c_size_t, vp]
        L.gravac_decompress_update.restype = i32
        L.gravac_decompress_update.argtypes = [vp, vp, vp, i32, i64, ctypes.c_float, vp, vp, ctypes.c_size_t, vp]
        L.gravac_decompress_accumulate_static.restype = i32
        L.gravac_decompress_accumulate_static.argtypes = [vp, vp, vp, i32, i64, vp, vp]
        L.gravac_decompress_workspace_bytes.restype = i32
        L.gravac_decompress_workspace_bytes.argtypes = [i32, i64, ctypes.POINTER(ctypes.c_size_t)]
        L.gravac_read_status.restype = i32
        L.gravac_read_status.argtypes = [vp, vp, vp]
        L.gravac_strerror.restype = ctypes.c_char_p
        L.gravac_strerror.argtypes = [i32]
        dp = ctypes.POINTER(dbl)
        L.gravac_controller_create.restype = i32
        L.gravac_controller_create.argtypes = [ctypes.POINTER(ControllerConfig), ctypes.POINTER(vp)]
        L.gravac_controller_destroy.restype = None
        L.gravac_controller_destroy.argtypes = [vp]
        L.gravac_controller_candidates.restype = i32
        L.gravac_controller_candidates.argtypes = [vp, dp, dp, dp]
        L.gravac_controller_decide.restype = i32
        L.gravac_controller_decide.argtypes = [vp, dbl, dbl, ctypes.POINTER(ctypes.c_int32), dp, dp]
        L.gravac_controller_finish_iteration.restype = i32
        L.gravac_controller_finish_iteration.argtypes = [vp, dbl, dp]
        L.gravac_controller_throughput.restype = i32
        L.gravac_controller_throughput.argtypes = [vp, dbl, dp]
        L.gravac_controller_iteration.restype = i64
        L.gravac_controller_iteration.argtypes = [vp]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().gravac_strerror(int(code)).decode()


def gravac_topk_count(n: int, cf: float) -> int:
    return int(lib().gravac_topk_count(int(n), float(cf)))


def gravac_workspace_bytes(n: int, n_cf: int, n_seg: int = 0) -> int:
    out = ctypes.c_size_t(0)
    rc = lib().gravac_workspace_bytes(int(n), int(n_cf), int(n_seg), ctypes.byref(out))
    if rc != OK:
        raise GravacError(rc, "gravac_workspace_bytes")
    return int(out.value)


def _stream_handle(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _dev_ptr(t, dtype) -> int:
    if t is None:
        return 0
    assert t.is_cuda and t.dtype == dtype and t.is_contiguous(), "expected a contiguous device tensor"
    return t.data_ptr()


class CallTimer:
    """Four torch events for ``gravac_compress_profiled``: ``call_ms()`` and ``pass_ms()`` after a call."""

    def __init__(self):
        self.events = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        for e in self.events:       # torch creates the HIP event on the first record
            e.record()
        torch.cuda.synchronize()
        self.struct = ProfileEvents(*[ctypes.c_void_p(int(e.cuda_event)) for e in self.events])
        assert all(int(e.cuda_event) != 0 for e in self.events)

    def call_ms(self) -> float:
        self.events[3].synchronize()
        return self.events[0].elapsed_time(self.events[3])

    def pass_ms(self) -> float:
        self.events[3].synchronize()
        return self.events[1].elapsed_time(self.events[2])


def gravac_compress(grad, residual, cf_list, commit=0, seg_offsets=None, *, out_idx, out_val,
                    out_count=None, out_stats, workspace, flags=0, stream=None, timer=None) -> None:
    """``gravac_compress`` of the C ABI on torch device tensors (asynchronous on ``stream``); with a ``CallTimer``,
    ``gravac_compress_profiled``."""
    cfs = np.ascontiguousarray(np.asarray(cf_list, dtype=np.float64))
    if seg_offsets is None:
        seg_ptr, n_seg = None, 0
    else:
        seg = np.ascontiguousarray(np.asarray(seg_offsets, dtype=np.int64))
        seg_ptr, n_seg = seg.ctypes.data_as(ctypes.c_void_p), seg.size - 1
    args = (_dev_ptr(grad, torch.float32), _dev_ptr(residual, torch.float32), grad.numel(),
            cfs.ctypes.data_as(ctypes.c_void_p), cfs.size, int(commit), seg_ptr, n_seg,
            _dev_ptr(out_idx, torch.int32), _dev_ptr(out_val, torch.float32), out_idx.numel(),
            _dev_ptr(out_count, torch.int64), _dev_ptr(out_stats, torch.float64),
            workspace.data_ptr(), workspace.numel() * workspace.element_size(), int(flags), _stream_handle(stream))
    if timer is None:
        rc = lib().gravac_compress(*args)
    else:
        rc = lib().gravac_compress_profiled(*args, ctypes.byref(timer.struct))
    if rc != OK:
        raise GravacError(rc, "gravac_compress")


def gravac_randomk_compress(grad, residual, cf_list, seed, commit=0, seg_offsets=None, *, out_idx, out_val,
                            out_count=None, out_stats, workspace, flags=0, stream=None) -> None:
    """``gravac_randomk_compress`` of the C ABI on torch device tensors (asynchronous on ``stream``)."""
    cfs = np.ascontiguousarray(np.asarray(cf_list, dtype=np.float64))
    if seg_offsets is None:
        seg_ptr, n_seg = None, 0
    else:
        seg = np.ascontiguousarray(np.asarray(seg_offsets, dtype=np.int64))
        seg_ptr, n_seg = seg.ctypes.data_as(ctypes.c_void_p), seg.size - 1
    rc = lib().gravac_randomk_compress(
        _dev_ptr(grad, torch.float32), _dev_ptr(residual, torch.float32), grad.numel(),
        cfs.ctypes.data_as(ctypes.c_void_p), cfs.size, int(commit), int(seed) & 0xFFFFFFFFFFFFFFFF, seg_ptr, n_seg,
        _dev_ptr(out_idx, torch.int32), _dev_ptr(out_val, torch.float32), out_idx.numel(),
        _dev_ptr(out_count, torch.int64), _dev_ptr(out_stats, torch.float64),
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), int(flags), _stream_handle(stream))
    if rc != OK:
        raise GravacError(rc, "gravac_randomk_compress")


def gravac_threshold_compress(grad, residual, tau, *, out_idx, out_val, out_count, out_stats, workspace, stream=None) -> None:
    """``gravac_threshold_compress`` of the C ABI on torch device tensors (asynchronous on ``stream``)."""
    rc = lib().gravac_threshold_compress(
        _dev_ptr(grad, torch.float32), _dev_ptr(residual, torch.float32), grad.numel(), ctypes.c_float(tau),
        _dev_ptr(out_idx, torch.int32), _dev_ptr(out_val, torch.float32), out_idx.numel(),
        _dev_ptr(out_count, torch.int64), _dev_ptr(out_stats, torch.float64),
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc != OK:
        raise GravacError(rc, "gravac_threshold_compress")


def gravac_recompress(idx1, val1, cf_rel, seg_counts=None, residual=None, *, out_idx, out_val, out_count=None,
                      out_stats, workspace, flags=0, stream=None) -> None:
    """``gravac_recompress`` of the C ABI on torch device tensors (asynchronous on ``stream``)."""
    if seg_counts is None:
        cnt_ptr, n_seg = None, 0
    else:
        cnt = np.ascontiguousarray(np.asarray(seg_counts, dtype=np.int64))
        cnt_ptr, n_seg = cnt.ctypes.data_as(ctypes.c_void_p), cnt.size
    rc = lib().gravac_recompress(
        _dev_ptr(idx1, torch.int32), _dev_ptr(val1, torch.float32), idx1.numel(), float(cf_rel), cnt_ptr, n_seg,
        _dev_ptr(residual, torch.float32), 0 if residual is None else residual.numel(),
        _dev_ptr(out_idx, torch.int32), _dev_ptr(out_val, torch.float32), out_idx.numel(),
        _dev_ptr(out_count, torch.int64), _dev_ptr(out_stats, torch.float64),
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), int(flags), _stream_handle(stream))
    if rc != OK:
        raise GravacError(rc, "gravac_recompress")


def gravac_commit(idx, residual, *, stream=None) -> None:
    """``gravac_commit`` of the C ABI: residual[idx] = +0."""
    rc = lib().gravac_commit(_dev_ptr(idx, torch.int32), idx.numel(), _dev_ptr(residual, torch.float32),
                             residual.numel(), _stream_handle(stream))
    if rc != OK:
        raise GravacError(rc, "gravac_commit")


def gravac_decompress_workspace_bytes(W: int, n: int) -> int:
    out = ctypes.c_size_t(0)
    rc = lib().gravac_decompress_workspace_bytes(int(W), int(n), ctypes.byref(out))
    if rc != OK:
        raise GravacError(rc, "gravac_decompress_workspace_bytes")
    return int(out.value)


def gravac_decompress_accumulate(idx, val, counts, dense_out, *, workspace=None, stream=None) -> None:
    """``gravac_decompress_accumulate`` of the C ABI on torch device tensors (``workspace``: a uint8 device
    tensor of at least ``gravac_decompress_workspace_bytes`` bytes, or None)."""
    cnt = np.ascontiguousarray(np.asarray(counts, dtype=np.int64))
    rc = lib().gravac_decompress_accumulate(
        _dev_ptr(idx, torch.int32), _dev_ptr(val, torch.float32), cnt.ctypes.data_as(ctypes.c_void_p),
        cnt.size, dense_out.numel(), _dev_ptr(dense_out, torch.float32),
        0 if workspace is None else workspace.data_ptr(),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc != OK:
        raise GravacError(rc, "gravac_decompress_accumulate")


def gravac_decompress_update(idx, val, counts, alpha, params, *, workspace=None, stream=None) -> None:
    """``gravac_decompress_update`` of the C ABI on torch device tensors: ``params[idx] += alpha * val`` pair by
    pair, workers in order (``workspace`` as for ``gravac_decompress_accumulate``)."""
    cnt = np.ascontiguousarray(np.asarray(counts, dtype=np.int64))
    rc = lib().gravac_decompress_update(
        _dev_ptr(idx, torch.int32), _dev_ptr(val, torch.float32), cnt.ctypes.data_as(ctypes.c_void_p),
        cnt.size, params.numel(), ctypes.c_float(alpha), _dev_ptr(params, torch.float32),
        0 if workspace is None else workspace.data_ptr(),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc != OK:
        raise GravacError(rc, "gravac_decompress_update")


def gravac_decompress_accumulate_static(idx, val, counts, dense_out, *, stream=None) -> None:
    """``gravac_decompress_accumulate_static`` of the C ABI: the same on the library's own static scratch."""
    cnt = np.ascontiguousarray(np.asarray(counts, dtype=np.int64))
    rc = lib().gravac_decompress_accumulate_static(
        _dev_ptr(idx, torch.int32), _dev_ptr(val, torch.float32), cnt.ctypes.data_as(ctypes.c_void_p),
        cnt.size, dense_out.numel(), _dev_ptr(dense_out, torch.float32), _stream_handle(stream))
    if rc != OK:
        raise GravacError(rc, "gravac_decompress_accumulate_static")


def gravac_read_status(workspace, stream=None) -> dict:
    out = (ctypes.c_int32 * 8)()
    rc = lib().gravac_read_status(workspace.data_ptr(), _stream_handle(stream), out)
    if rc != OK:
        raise GravacError(rc, "gravac_read_status")
    return {"any_fallback": int(out[0]), "fallback_segments": int(out[1]), "internal_error": int(out[2]),
            "segments": int(out[3]), "narrow_fallback_segments": int(out[4])}


# --------------------------------------------------------------------------
# convenience: allocate outputs and workspace with torch, call, return tensors
# --------------------------------------------------------------------------

class Compressor:
    """Owns the workspace and output buffers for repeated calls on one gradient shape."""

    def __init__(self, n: int, cf_list, commit: int = 0, seg_offsets=None, device="cuda"):
        self.n = int(n)
        self.cfs = [float(c) for c in cf_list]
        self.commit = int(commit)
        self.seg = None if seg_offsets is None else np.asarray(seg_offsets, dtype=np.int64)
        n_seg = 0 if self.seg is None else self.seg.size - 1
        sizes = [self.n] if self.seg is None else np.diff(self.seg).tolist()
        self.k_total = sum(gravac_topk_count(int(s), self.cfs[self.commit]) for s in sizes)
        self.rows = max(n_seg, 1)
        self.workspace = torch.empty(gravac_workspace_bytes(self.n, len(self.cfs), n_seg), dtype=torch.uint8,
                                     device=device)
        self.out_idx = torch.empty(self.k_total, dtype=torch.int32, device=device)
        self.out_val = torch.empty(self.k_total, dtype=torch.float32, device=device)
        self.out_count = torch.zeros(1, dtype=torch.int64, device=device)
        self.out_stats = torch.zeros(self.rows, len(self.cfs), 4, dtype=torch.float64, device=device)

    def __call__(self, grad, residual, flags=0, stream=None, timer=None):
        gravac_compress(grad, residual, self.cfs, self.commit, self.seg, out_idx=self.out_idx,
                        out_val=self.out_val, out_count=self.out_count, out_stats=self.out_stats,
                        workspace=self.workspace, flags=flags, stream=stream, timer=timer)
        return self.out_idx, self.out_val, self.out_stats

    def randomk(self, grad, residual, seed, flags=0, stream=None):
        """The same buffers with Random-k instead of Top-k."""
        gravac_randomk_compress(grad, residual, self.cfs, seed, self.commit, self.seg, out_idx=self.out_idx,
                                out_val=self.out_val, out_count=self.out_count, out_stats=self.out_stats,
                                workspace=self.workspace, flags=flags, stream=stream)
        return self.out_idx, self.out_val, self.out_stats

    def status(self) -> dict:
        return gravac_read_status(self.workspace)


class Controller:
    """The host-side adaptive-compression controller of the C ABI (``gravac_controller_*``)."""

    def __init__(self, theta_min, theta_max, epsilon, omega, window, policy=POLICY_GEOMETRIC, theta_s=2.0,
                 alpha=0.32, samples_per_iteration=1.0):
        cfg = ControllerConfig(float(theta_min), float(theta_max), float(epsilon), float(omega), float(theta_s),
                               float(alpha), float(samples_per_iteration), int(window), int(policy), 0)
        h = ctypes.c_void_p()
        rc = lib().gravac_controller_create(ctypes.byref(cfg), ctypes.byref(h))
        if rc != OK:
            raise GravacError(rc, "gravac_controller_create")
        self._h = h

    def close(self):
        if self._h:
            lib().gravac_controller_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def candidates(self):
        """(theta_min, theta_c, theta_c / theta_min) for the coming iteration."""
        a, b, c = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
        rc = lib().gravac_controller_candidates(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
        if rc != OK:
            raise GravacError(rc, "gravac_controller_candidates")
        return a.value, b.value, c.value

    def decide(self, gain_min, gain_c):
        """(choice, delta_min, delta_c)."""
        ch, a, b = ctypes.c_int32(), ctypes.c_double(), ctypes.c_double()
        rc = lib().gravac_controller_decide(self._h, float(gain_min), float(gain_c), ctypes.byref(ch),
                                            ctypes.byref(a), ctypes.byref(b))
        if rc != OK:
            raise GravacError(rc, "gravac_controller_decide")
        return ch.value, a.value, b.value

    def finish_iteration(self, t_iter):
        s = ctypes.c_double()
        rc = lib().gravac_controller_finish_iteration(self._h, float(t_iter), ctypes.byref(s))
        if rc != OK:
            raise GravacError(rc, "gravac_controller_finish_iteration")
        return s.value

    def throughput(self, cf):
        """T_compress[cf], or None if that CF has no entry yet."""
        t = ctypes.c_double()
        rc = lib().gravac_controller_throughput(self._h, float(cf), ctypes.byref(t))
        return t.value if rc == OK else None

    @property
    def iteration(self):
        return int(lib().gravac_controller_iteration(self._h))
