"""GPU test of gravac_decompress_accumulate_static, the entry point that allocates nothing: its output against
gravac_decompress_accumulate with a caller workspace (same kernels, the boundaries in the library's static scratch),
bit for bit, on two calls in a row, the second with a smaller input (the scratch keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2305_12201_amd import binding

pytestmark = pytest.mark.gpu


def _messages(n, ks, seed):
    rng = np.random.default_rng(seed)
    idx = np.concatenate([np.sort(rng.choice(n, k, replace=False)) for k in ks]).astype(np.int32)
    val = rng.standard_normal(idx.size).astype(np.float32)
    dense = rng.standard_normal(n).astype(np.float32)
    return idx, val, dense


def _both(n, ks, seed):
    idx, val, dense = _messages(n, ks, seed)
    di, dv = torch.from_numpy(idx).cuda(), torch.from_numpy(val).cuda()
    cnt = np.asarray(ks, dtype=np.int64)
    L = binding.lib()
    stream = torch.cuda.current_stream().cuda_stream
    # the existing entry point, through the C ABI, with a workspace of the caller
    want = torch.from_numpy(dense).cuda()
    ws = torch.empty(binding.gravac_decompress_workspace_bytes(len(ks), n), dtype=torch.uint8, device="cuda")
    rc = L.gravac_decompress_accumulate(di.data_ptr(), dv.data_ptr(), cnt.ctypes.data_as(ctypes.c_void_p), len(ks), n,
                                        want.data_ptr(), ws.data_ptr(), ws.numel(), stream)
    assert rc == 0
    # the entry point that allocates nothing
    got = torch.from_numpy(dense).cuda()
    rc = L.gravac_decompress_accumulate_static(di.data_ptr(), dv.data_ptr(), cnt.ctypes.data_as(ctypes.c_void_p),
                                               len(ks), n, got.data_ptr(), stream)
    assert rc == 0
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.cpu().numpy().view(np.uint32)), (n, ks)
    # and against plain numpy adds, worker by worker
    ref = dense.copy()
    at = 0
    for k in ks:
        ref[idx[at:at + k]] += val[at:at + k]
        at += k
    assert np.array_equal(got.cpu().numpy().view(np.uint32), ref.view(np.uint32)), (n, ks)


def test_static_scratch_two_calls_second_smaller():
    _both(3_000_017, [40_000, 0, 90_000, 12_345, 7, 250_000, 3000, 66_666], seed=11)   # 367 tiles, 8 workers
    _both(100_003, [5000, 100, 20_000], seed=12)                                        # 13 tiles, 3 workers
    _both(8192 * 70 + 5, [300] * 70, seed=13)                                           # more than 64 workers: two groups


def test_static_scratch_limit_and_arguments():
    L = binding.lib()
    d = torch.zeros(16, dtype=torch.float32, device="cuda")
    i = torch.zeros(4, dtype=torch.int32, device="cuda")
    v = torch.zeros(4, dtype=torch.float32, device="cuda")
    cnt = np.array([1] * 64, dtype=np.int64)
    # 64 workers on 2^31 - 1 elements: 64 * 262145 boundaries do not fit the static scratch; nothing is launched
    rc = L.gravac_decompress_accumulate_static(i.data_ptr(), v.data_ptr(), cnt.ctypes.data_as(ctypes.c_void_p), 64,
                                               2**31 - 1, d.data_ptr(), 0)
    assert rc == binding.ERR_STATIC_LIMIT
    assert binding.gravac_decompress_workspace_bytes(8, 1_000_000_000) <= binding.STATIC_SCRATCH_BYTES
    rc = L.gravac_decompress_accumulate_static(i.data_ptr(), v.data_ptr(), cnt.ctypes.data_as(ctypes.c_void_p), 0, 16,
                                               d.data_ptr(), 0)
    assert rc == binding.ERR_INVALID_ARG
    torch.cuda.synchronize()
