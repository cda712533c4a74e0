"""ctypes front end of the CPU oracle (``gravac_oracle.c``).

TEST INFRASTRUCTURE ONLY.  The oracle is the plain single-threaded definition of
the GraVAC compression path (Sec. II-C Top-k, Sec. III-B error feedback and
compression gain, Alg. 1 residual update, Sec. III-A layerwise mode and
decompression).  Only the tests, the smoke check and the bench's ``cpu_baseline``
leg may import this module; the product package never does, and this module
imports nothing from the product package.

All arrays are host numpy arrays.  ``build()`` compiles the C file with gcc.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gravac_oracle.c")
_LIB = os.path.join(_HERE, "libgravac_oracle.so")

_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle (gcc, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c99", "-fPIC", "-shared",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        lib = ctypes.CDLL(_LIB)
        i64, dbl, i32 = ctypes.c_int64, ctypes.c_double, ctypes.c_int
        p = ctypes.c_void_p
        lib.oracle_k.restype = i64
        lib.oracle_k.argtypes = [i64, dbl]
        lib.oracle_compress.restype = i32
        lib.oracle_compress.argtypes = [p, p, i64, p, i32, i32, p, i32, p, p, i64, p, p]
        lib.oracle_decompress_accumulate.restype = i32
        lib.oracle_decompress_accumulate.argtypes = [p, p, p, i32, i64, p]
        lib.oracle_decompress_update.restype = i32
        lib.oracle_decompress_update.argtypes = [p, p, p, i32, i64, ctypes.c_float, p]
        lib.oracle_commit.restype = i32
        lib.oracle_commit.argtypes = [p, i64, p, i64]
        lib.oracle_splitmix64_first.restype = ctypes.c_uint64
        lib.oracle_splitmix64_first.argtypes = [ctypes.c_uint64]
        lib.oracle_randomk_priority.restype = ctypes.c_uint32
        lib.oracle_randomk_priority.argtypes = [ctypes.c_uint64, ctypes.c_uint32]
        lib.oracle_randomk_compress.restype = i32
        lib.oracle_randomk_compress.argtypes = [p, p, i64, p, i32, i32, ctypes.c_uint64, p, i32, p, p, i64, p, p]
        lib.oracle_threshold_compress.restype = i32
        lib.oracle_threshold_compress.argtypes = [p, p, i64, ctypes.c_float, p, p, i64, p, p]
        lib.oracle_recompress.restype = i32
        lib.oracle_recompress.argtypes = [p, p, i64, dbl, p, i64, p, i32, p, p, i64, p, p]
        _lib = lib
    return _lib


def topk_count(n: int, cf: float) -> int:
    """k = ceil(n / CF) clamped to [1, n] (Sec. II-C)."""
    return int(_load().oracle_k(int(n), float(cf)))


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def compress(grad: np.ndarray, residual: np.ndarray, cf_list, commit: int = 0, seg_offsets=None):
    """Run the oracle on host arrays.

    ``residual`` (float32, C-contiguous) is updated IN PLACE.  Returns
    ``(idx int32[k], val float32[k], stats float64[n_seg][n_cf][4])`` where a
    stats row is ``(||g_c||^2, ||g_ef||^2, gain, |acc| of the smallest selected)``.
    """
    lib = _load()
    assert grad.dtype == np.float32 and residual.dtype == np.float32
    assert grad.flags.c_contiguous and residual.flags.c_contiguous
    n = grad.size
    assert residual.size == n
    cfs = np.ascontiguousarray(np.asarray(cf_list, dtype=np.float64))
    n_cf = cfs.size
    if seg_offsets is None:
        off = None
        n_seg = 0
        rows = 1
        cap = topk_count(n, cfs[commit])
    else:
        off = np.ascontiguousarray(np.asarray(seg_offsets, dtype=np.int64))
        n_seg = off.size - 1
        rows = n_seg
        cap = sum(topk_count(int(off[t + 1] - off[t]), cfs[commit]) for t in range(n_seg))
    idx = np.empty(cap, dtype=np.int32)
    val = np.empty(cap, dtype=np.float32)
    stats = np.zeros((rows, n_cf, 4), dtype=np.float64)
    count = ctypes.c_int64(0)
    rc = lib.oracle_compress(_ptr(grad), _ptr(residual), n, _ptr(cfs), n_cf, int(commit),
                             _ptr(off) if off is not None else None, n_seg,
                             _ptr(idx), _ptr(val), cap, ctypes.byref(count), _ptr(stats))
    if rc != 0:
        raise RuntimeError(f"oracle_compress failed with code {rc}")
    assert count.value == cap
    return idx, val, stats


def decompress_accumulate(idx: np.ndarray, val: np.ndarray, counts, dense_out: np.ndarray) -> None:
    """dense_out[idx] += val, workers in order (Sec. III-A decompression), in place."""
    lib = _load()
    assert idx.dtype == np.int32 and val.dtype == np.float32 and dense_out.dtype == np.float32
    cnt = np.ascontiguousarray(np.asarray(counts, dtype=np.int64))
    rc = lib.oracle_decompress_accumulate(_ptr(np.ascontiguousarray(idx)), _ptr(np.ascontiguousarray(val)),
                                          _ptr(cnt), cnt.size, dense_out.size, _ptr(dense_out))
    if rc != 0:
        raise RuntimeError(f"oracle_decompress_accumulate failed with code {rc}")


def decompress_update(idx: np.ndarray, val: np.ndarray, counts, alpha: float, w: np.ndarray) -> None:
    """w[idx] += alpha * val pair by pair (product, then sum, each rounded to binary32), workers in order, in
    place: with alpha = -eta / W the update step of Alg. 1 applied straight from the W messages."""
    lib = _load()
    assert idx.dtype == np.int32 and val.dtype == np.float32 and w.dtype == np.float32
    cnt = np.ascontiguousarray(np.asarray(counts, dtype=np.int64))
    rc = lib.oracle_decompress_update(_ptr(np.ascontiguousarray(idx)), _ptr(np.ascontiguousarray(val)),
                                      _ptr(cnt), cnt.size, w.size, ctypes.c_float(alpha), _ptr(w))
    if rc != 0:
        raise RuntimeError(f"oracle_decompress_update failed with code {rc}")


def commit(idx: np.ndarray, residual: np.ndarray) -> None:
    """residual[idx] = +0 in place (Alg. 1, residual update of the message that was sent)."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    assert residual.dtype == np.float32 and residual.flags.c_contiguous
    rc = _load().oracle_commit(_ptr(idx), idx.size, _ptr(residual), residual.size)
    if rc != 0:
        raise RuntimeError(f"oracle_commit failed with code {rc}")


def recompress(idx1: np.ndarray, val1: np.ndarray, cf_rel: float, residual=None, seg_counts=None):
    """Second-level Top-k on a message (Sec. IV-C multi-level compression).

    Returns ``(idx int32[k2], val float32[k2], stats float64[n_seg][4])``.  ``residual`` (float32, the
    residual left by committing the level-1 message), if given, is updated IN PLACE to the residual
    of committing the level-2 message.
    """
    lib = _load()
    idx1 = np.ascontiguousarray(idx1, dtype=np.int32)
    val1 = np.ascontiguousarray(val1, dtype=np.float32)
    k1 = idx1.size
    if seg_counts is None:
        cnt, n_seg, rows = None, 0, 1
        cap = topk_count(k1, cf_rel)
    else:
        cnt = np.ascontiguousarray(np.asarray(seg_counts, dtype=np.int64))
        n_seg, rows = cnt.size, cnt.size
        cap = sum(topk_count(int(c), cf_rel) for c in cnt)
    out_idx = np.empty(cap, dtype=np.int32)
    out_val = np.empty(cap, dtype=np.float32)
    stats = np.zeros((rows, 4), dtype=np.float64)
    count = ctypes.c_int64(0)
    rc = lib.oracle_recompress(_ptr(idx1), _ptr(val1), k1, float(cf_rel),
                               _ptr(residual) if residual is not None else None,
                               residual.size if residual is not None else 0,
                               _ptr(cnt) if cnt is not None else None, n_seg,
                               _ptr(out_idx), _ptr(out_val), cap, ctypes.byref(count), _ptr(stats))
    if rc != 0:
        raise RuntimeError(f"oracle_recompress failed with code {rc}")
    assert count.value == cap
    return out_idx, out_val, stats


def splitmix64_first(seed: int) -> int:
    """First output of the SplitMix64 generator started at ``seed`` (the seed mixing of Random-k)."""
    return int(_load().oracle_splitmix64_first(int(seed) & 0xFFFFFFFFFFFFFFFF))


def randomk_priority(seed: int, i: int) -> int:
    """Priority of index i under the seed (Random-k; the keyed 31-bit bijection of the oracle's header)."""
    return int(_load().oracle_randomk_priority(int(seed) & 0xFFFFFFFFFFFFFFFF, int(i)))


def randomk_compress(grad: np.ndarray, residual: np.ndarray, cf_list, seed: int, commit: int = 0, seg_offsets=None):
    """Random-k with error feedback (Sec. II-C); same conventions as ``compress``.

    Returns ``(idx, val, stats)``; a stats row is ``(||g_c||^2, ||g_ef||^2, gain, lowest selected priority)``.
    """
    lib = _load()
    assert grad.dtype == np.float32 and residual.dtype == np.float32
    assert grad.flags.c_contiguous and residual.flags.c_contiguous
    n = grad.size
    cfs = np.ascontiguousarray(np.asarray(cf_list, dtype=np.float64))
    n_cf = cfs.size
    if seg_offsets is None:
        off, n_seg, rows = None, 0, 1
        cap = topk_count(n, cfs[commit])
    else:
        off = np.ascontiguousarray(np.asarray(seg_offsets, dtype=np.int64))
        n_seg = rows = off.size - 1
        cap = sum(topk_count(int(off[t + 1] - off[t]), cfs[commit]) for t in range(n_seg))
    idx = np.empty(cap, dtype=np.int32)
    val = np.empty(cap, dtype=np.float32)
    stats = np.zeros((rows, n_cf, 4), dtype=np.float64)
    count = ctypes.c_int64(0)
    rc = lib.oracle_randomk_compress(_ptr(grad), _ptr(residual), n, _ptr(cfs), n_cf, int(commit),
                                     int(seed) & 0xFFFFFFFFFFFFFFFF, _ptr(off) if off is not None else None, n_seg,
                                     _ptr(idx), _ptr(val), cap, ctypes.byref(count), _ptr(stats))
    if rc != 0:
        raise RuntimeError(f"oracle_randomk_compress failed with code {rc}")
    assert count.value == cap
    return idx, val, stats


def threshold_compress(grad: np.ndarray, residual: np.ndarray, tau: float, capacity=None):
    """Threshold sparsifier with error feedback (Sec. II-C, the selection rule given for DGC): keep |acc| >= tau.

    ``residual`` is updated IN PLACE.  Returns ``(idx, val, stats float64[4], count)``; a stats row is
    ``(||g_c||^2, ||g_ef||^2, gain, tau)``.  With ``capacity`` smaller than the number of kept entries the message
    is empty (``idx.size == 0``), the residual holds acc and ``count`` still says how many would have been kept.
    """
    lib = _load()
    assert grad.dtype == np.float32 and residual.dtype == np.float32
    assert grad.flags.c_contiguous and residual.flags.c_contiguous and residual.size == grad.size
    n = grad.size
    cap = n if capacity is None else int(capacity)
    idx = np.empty(cap, dtype=np.int32)
    val = np.empty(cap, dtype=np.float32)
    stats = np.zeros(4, dtype=np.float64)
    count = ctypes.c_int64(0)
    rc = lib.oracle_threshold_compress(_ptr(grad), _ptr(residual), n, ctypes.c_float(tau), _ptr(idx), _ptr(val), cap,
                                       ctypes.byref(count), _ptr(stats))
    if rc == -2:                              # capacity: nothing emitted
        return idx[:0], val[:0], stats, int(count.value)
    if rc != 0:
        raise RuntimeError(f"oracle_threshold_compress failed with code {rc}")
    return idx[:count.value].copy(), val[:count.value].copy(), stats, int(count.value)
