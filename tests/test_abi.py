"""CPU-side checks of the C ABI: the library loads, exports what the header declares, validates arguments."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2305_12201_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = set()
    for header in ("gravac.h", "gravac_profile.h", "gravac_controller.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(gravac_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTS)
    L = binding.lib()
    for name in names:
        assert getattr(L, name) is not None


def test_topk_count_matches_printed_values():
    rows = []
    for fn in ("cf_fraction.txt", "k_values.txt"):
        for line in open(os.path.join(ROOT, "tests", "golden", fn)):
            if line.strip() and not line.startswith("#"):
                rows.append(line.split())
    for n, cf, k in rows:
        assert binding.gravac_topk_count(int(n), float(cf)) == int(k)
    assert binding.gravac_topk_count(10, 1.5) == 7
    assert binding.gravac_topk_count(3, 1000) == 1
    assert binding.gravac_topk_count(0, 10) == -1
    assert binding.gravac_topk_count(10, 0.5) == -1
    assert binding.gravac_topk_count(10, float("inf")) == -1
    assert binding.gravac_topk_count(10, float("nan")) == -1


def test_workspace_bytes():
    a = binding.gravac_workspace_bytes(1 << 20, 1, 0)
    b = binding.gravac_workspace_bytes(1 << 21, 1, 0)
    c = binding.gravac_workspace_bytes(1 << 20, 3, 0)
    d = binding.gravac_workspace_bytes(1 << 20, 1, 314)
    assert 8 * (1 << 20) <= a < b and a < c and a < d
    assert binding.gravac_workspace_bytes(1 << 20, 1, 1) == a      # one segment is the flat case
    for bad in ((0, 1, 0), (1 << 31, 1, 0), (100, 0, 0), (100, 9, 0), (100, 1, -1), (5, 1, 6)):
        with pytest.raises(binding.GravacError) as e:
            binding.gravac_workspace_bytes(*bad)
        assert e.value.code == binding.ERR_INVALID_ARG


def _call(L, grad=0x1000, res=0x2000, n=100, cfs=(10.0,), commit=0, seg=None, out_idx=0x3000, out_val=0x4000,
          cap=100, out_stats=0x5000, ws=0x10000, ws_bytes=1 << 40):
    """Argument validation happens before any pointer is touched, so fake addresses are safe here."""
    cf = np.asarray(cfs, dtype=np.float64)
    segp, nseg = (None, 0)
    if seg is not None:
        s = np.asarray(seg, dtype=np.int64)
        segp, nseg = s.ctypes.data_as(ctypes.c_void_p), s.size - 1
    return L.gravac_compress(grad, res, n, cf.ctypes.data_as(ctypes.c_void_p), cf.size, commit, segp, nseg,
                             out_idx, out_val, cap, None, out_stats, ws, ws_bytes, 0, None)


def test_compress_rejects_bad_arguments_without_touching_memory():
    L = binding.lib()
    E = binding
    assert _call(L, grad=0) == E.ERR_INVALID_ARG
    assert _call(L, res=0) == E.ERR_INVALID_ARG
    assert _call(L, out_idx=0) == E.ERR_INVALID_ARG
    assert _call(L, out_stats=0) == E.ERR_INVALID_ARG
    assert _call(L, grad=0x1002) == E.ERR_INVALID_ARG            # not at a float boundary
    assert L.gravac_compress(0x1000, 0x2000, 100, np.asarray([10.0]).ctypes.data_as(ctypes.c_void_p), 1, 0, None, 0,
                             0x3000, 0x4000, 100, None, 0x5000, 0x10000, 1 << 40, 6, None) == E.ERR_INVALID_ARG  # unknown flag
    assert _call(L, n=0) == E.ERR_INVALID_ARG
    assert _call(L, n=1 << 31) == E.ERR_INVALID_ARG
    assert _call(L, cfs=(0.5,)) == E.ERR_INVALID_ARG
    assert _call(L, cfs=(float("nan"),)) == E.ERR_INVALID_ARG
    assert _call(L, cfs=(float("inf"),)) == E.ERR_INVALID_ARG
    assert _call(L, cfs=(10.0,) * 9) == E.ERR_INVALID_ARG
    assert _call(L, commit=1) == E.ERR_INVALID_ARG
    assert _call(L, commit=-1) == E.ERR_INVALID_ARG
    assert _call(L, seg=[0, 50, 50, 100]) == E.ERR_INVALID_ARG   # not strictly increasing
    assert _call(L, seg=[1, 50, 100]) == E.ERR_INVALID_ARG       # does not start at 0
    assert _call(L, seg=[0, 50, 99]) == E.ERR_INVALID_ARG        # does not end at n
    assert _call(L, cap=9) == E.ERR_CAPACITY                     # k = 10
    assert _call(L, seg=[0, 50, 100], cap=9) == E.ERR_CAPACITY   # 5 + 5
    assert _call(L, ws=0) == E.ERR_WORKSPACE
    assert _call(L, ws=0x10010) == E.ERR_WORKSPACE               # not 256-byte aligned
    assert _call(L, ws_bytes=1024) == E.ERR_WORKSPACE


def test_decompress_rejects_bad_arguments():
    L = binding.lib()
    cnt = np.asarray([5, -1], dtype=np.int64)
    p = cnt.ctypes.data_as(ctypes.c_void_p)
    assert L.gravac_decompress_accumulate(0x1000, 0x2000, p, 2, 100, 0x3000, None, 0, None) == binding.ERR_INVALID_ARG
    cnt[1] = 1
    assert L.gravac_decompress_accumulate(0x1000, 0x2000, p, 0, 100, 0x3000, None, 0, None) == binding.ERR_INVALID_ARG
    assert L.gravac_decompress_accumulate(0x1000, 0x2000, p, 2, 0, 0x3000, None, 0, None) == binding.ERR_INVALID_ARG
    assert L.gravac_decompress_accumulate(0x1000, 0x2000, p, 2, 100, 0, None, 0, None) == binding.ERR_INVALID_ARG
    assert L.gravac_decompress_accumulate(0, 0x2000, p, 2, 100, 0x3000, None, 0, None) == binding.ERR_INVALID_ARG
    assert L.gravac_decompress_accumulate(0x1000, 0x2000, None, 2, 100, 0x3000, None, 0, None) == binding.ERR_INVALID_ARG
    a = ctypes.c_float(-0.1)
    assert L.gravac_decompress_update(0x1000, 0x2000, p, 2, 100, a, 0, None, 0, None) == binding.ERR_INVALID_ARG
    assert L.gravac_decompress_update(0x1000, 0x2000, p, 0, 100, a, 0x3000, None, 0, None) == binding.ERR_INVALID_ARG
    assert L.gravac_decompress_update(0x1000, 0x2000, p, 2, 0, a, 0x3000, None, 0, None) == binding.ERR_INVALID_ARG
    assert L.gravac_decompress_update(0, 0x2000, p, 2, 100, a, 0x3000, None, 0, None) == binding.ERR_INVALID_ARG
    assert L.gravac_decompress_update(0x1000, 0x2000, None, 2, 100, a, 0x3000, None, 0, None) == binding.ERR_INVALID_ARG
    assert L.gravac_decompress_update(0x1000, 0x2000, p, 2, 100, a, 0x3000, 0x4001, 1 << 20, None) == binding.ERR_WORKSPACE
    assert L.gravac_decompress_update(0x1000, 0x2000, p, 2, 100, a, 0x3000, 0x4000, 8, None) == binding.ERR_WORKSPACE


def test_strerror():
    assert binding.strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -5, -6):
        assert binding.strerror(code) and "unknown" not in binding.strerror(code)
    assert "unknown" in binding.strerror(-99)
