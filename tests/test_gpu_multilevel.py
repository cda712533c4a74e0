"""GPU parity of multi-level compression (Sec. IV-C): gravac_recompress against the CPU oracle, and against a
direct compression at the higher CF (the identity the method relies on), through the C ABI.

Indices, values and residuals bit-exact; statistics within 1e-5 relative.
"""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2305_12201_amd import binding, workloads
from tests.gpu_util import STAT_RTOL, gpu_compress, oracle_compress

pytestmark = pytest.mark.gpu

FB = binding.FLAG_FORCE_FALLBACK


def gpu_recompress(idx1, val1, cf_rel, residual=None, seg_counts=None, flags=0):
    """Run gravac_recompress on host arrays; returns (idx, val, stats, residual or None, status)."""
    k1 = idx1.size
    n_seg = 0 if seg_counts is None else len(seg_counts)
    counts = [k1] if seg_counts is None else list(seg_counts)
    k2 = sum(binding.gravac_topk_count(int(c), cf_rel) for c in counts)
    di = torch.from_numpy(idx1).cuda()
    dv = torch.from_numpy(val1).cuda()
    dr = None if residual is None else torch.from_numpy(residual.copy()).cuda()
    ws = torch.empty(binding.gravac_workspace_bytes(k1, 1, n_seg), dtype=torch.uint8, device="cuda")
    out_idx = torch.full((k2,), -1, dtype=torch.int32, device="cuda")
    out_val = torch.full((k2,), float("nan"), dtype=torch.float32, device="cuda")
    out_count = torch.zeros(1, dtype=torch.int64, device="cuda")
    out_stats = torch.zeros(max(n_seg, 1), 4, dtype=torch.float64, device="cuda")
    binding.gravac_recompress(di, dv, cf_rel, seg_counts, dr, out_idx=out_idx, out_val=out_val, out_count=out_count,
                              out_stats=out_stats, workspace=ws, flags=flags)
    torch.cuda.synchronize()
    st = binding.gravac_read_status(ws)
    assert st["internal_error"] == 0
    assert int(out_count.item()) == k2
    assert np.array_equal(di.cpu().numpy(), idx1) and np.array_equal(dv.cpu().numpy().view(np.uint32),
                                                                    val1.view(np.uint32)), "level-1 message modified"
    return (out_idx.cpu().numpy(), out_val.cpu().numpy(), out_stats.cpu().numpy(),
            None if dr is None else dr.cpu().numpy(), st)


def assert_recompress_same(gpu, ref, ref_res, what=""):
    gi, gv, gs, gr = gpu[:4]
    oi, ov, os_ = ref
    assert np.array_equal(gi, oi), f"{what}: indices differ at {np.nonzero(gi != oi)[0][:5]}"
    assert np.array_equal(gv.view(np.uint32), ov.view(np.uint32)), f"{what}: values differ"
    if ref_res is not None:
        assert np.array_equal(gr.view(np.uint32), ref_res.view(np.uint32)), \
            f"{what}: residual differs at {np.nonzero(gr.view(np.uint32) != ref_res.view(np.uint32))[0][:5]}"
    assert gs.shape == os_.shape
    assert np.array_equal(gs[..., 3], os_[..., 3]), what
    np.testing.assert_allclose(gs[..., :3], os_[..., :3], rtol=STAT_RTOL, atol=0, err_msg=what)


def check_recompress(idx1, val1, cf_rel, residual=None, seg_counts=None, flags=0, what=""):
    gpu = gpu_recompress(idx1, val1, cf_rel, residual, seg_counts, flags)
    ref_res = None if residual is None else residual.copy()
    ref = oracle.recompress(idx1, val1, cf_rel, ref_res, seg_counts)
    assert_recompress_same(gpu, ref, ref_res, what)
    return gpu


@pytest.mark.parametrize("flags", [0, FB])
def test_two_levels_equal_direct_compression(flags):
    # level 1 at CF 10 on the GPU, level 2 at relative CF 10 on its message: the same message, residual and
    # threshold as a direct compression at CF 100; the product of the two gains is the direct gain
    n = 1_000_000                                       # ceil(ceil(n/10)/10) == ceil(n/100)
    g = workloads.normal_gradient(n, 1e-3, seed=301)
    r0 = workloads.normal_gradient(n, 3e-4, seed=302)
    i1, v1, s1, r1, _ = gpu_compress(g, r0, [10.0], flags=flags)
    gpu = check_recompress(i1, v1, 10.0, residual=r1, flags=flags, what="level 2 of 10x10")
    di, dv, ds, dr = oracle_compress(g, r0, [100.0])
    assert np.array_equal(gpu[0], di) and np.array_equal(gpu[1].view(np.uint32), dv.view(np.uint32))
    assert np.array_equal(gpu[3].view(np.uint32), dr.view(np.uint32))
    assert gpu[2][0, 3] == ds[0, 0, 3]
    np.testing.assert_allclose(s1[0, 0, 2] * gpu[2][0, 2], ds[0, 0, 2], rtol=STAT_RTOL)


@pytest.mark.parametrize("k1", [1, 2, 3, 63, 64, 65, 1023, 4096, 4097, 8193, 100_003, 1_048_577])
def test_ragged_message_sizes(k1):
    rng = np.random.default_rng(400 + k1)
    n = 4 * k1 + 7
    idx1 = np.sort(rng.choice(n, size=k1, replace=False)).astype(np.int32)
    val1 = (rng.standard_normal(k1) * 1e-3).astype(np.float32)
    res = (rng.standard_normal(n) * 1e-5).astype(np.float32)
    res[idx1] = 0.0
    for cf_rel in (1.0, 2.5, 10.0, 1000.0):
        check_recompress(idx1, val1, cf_rel, residual=res, what=f"k1={k1} cf_rel={cf_rel}")
    check_recompress(idx1, val1, 10.0, residual=None, what=f"k1={k1} no residual")


def test_ties_signed_zeros_and_specials():
    rng = np.random.default_rng(410)
    k1, n = 50_000, 400_000
    idx1 = np.sort(rng.choice(n, size=k1, replace=False)).astype(np.int32)
    val1 = rng.choice(np.array([0.0, -0.0, 1e-3, -1e-3, 2e-3, 1e-40, -1e-40], np.float32), size=k1)
    val1[100] = np.inf
    val1[200] = -np.inf
    val1[300] = np.nan
    res = np.zeros(n, np.float32)
    for cf_rel in (2.0, 7.0, 100.0):
        check_recompress(idx1, val1, cf_rel, residual=res, what=f"ties cf_rel={cf_rel}")
        check_recompress(idx1, val1, cf_rel, residual=res, flags=FB, what=f"ties exact route cf_rel={cf_rel}")


def test_out_of_range_indices_are_not_restored():
    rng = np.random.default_rng(420)
    k1, n = 10_000, 50_000
    idx1 = np.sort(rng.choice(2 * n, size=k1, replace=False)).astype(np.int32) - n // 2   # some < 0, some >= n
    val1 = (rng.standard_normal(k1)).astype(np.float32)
    res = np.full(n, 0.25, np.float32)
    gpu = gpu_recompress(idx1, val1, 10.0, residual=res)
    oi, ov, _ = oracle.recompress(idx1, val1, 10.0)
    assert np.array_equal(gpu[0], oi) and np.array_equal(gpu[1], ov)
    expect = res.copy()
    ok = (idx1 >= 0) & (idx1 < n)
    expect[idx1[ok]] = val1[ok]
    sel = oi[(oi >= 0) & (oi < n)]
    expect[sel] = 0.0
    assert np.array_equal(gpu[3].view(np.uint32), expect.view(np.uint32))


@pytest.mark.parametrize("flags", [0, FB])
def test_layerwise_two_levels(flags):
    sizes = [64, 1, 4096, 37, 100_003, 2, 9408, 1000, 4097, 8191, 3, 250_001, 5, 1_200_000]
    off = workloads.offsets_of(sizes)
    n = int(off[-1])
    g = workloads.resnet_like_gradient(n, seed=431)
    r0 = workloads.normal_gradient(n, 1e-5, seed=432)
    i1, v1, s1, r1, _ = gpu_compress(g, r0, [10.0], seg=off, flags=flags)
    counts = [binding.gravac_topk_count(s, 10.0) for s in sizes]
    assert sum(counts) == i1.size
    gpu = check_recompress(i1, v1, 10.0, residual=r1, seg_counts=counts, flags=flags, what="layerwise level 2")
    # tensors whose two-level k equals the direct k: the same entries as a direct compression at CF 100
    di, dv, ds, dr = oracle_compress(g, r0, [100.0], seg=off)
    same_k = [binding.gravac_topk_count(c, 10.0) == binding.gravac_topk_count(s, 100.0) for c, s in zip(counts, sizes)]
    assert all(same_k), "sizes were chosen so that both routes give the same k per tensor"
    assert np.array_equal(gpu[0], di) and np.array_equal(gpu[1].view(np.uint32), dv.view(np.uint32))
    assert np.array_equal(gpu[3].view(np.uint32), dr.view(np.uint32))


def test_three_levels_chain():
    # CF 10 -> 100 -> 1000 in three calls, residual handed from call to call, against direct compression at 1000
    n = 2_000_000
    g = workloads.normal_gradient(n, 1e-3, seed=441)
    r0 = workloads.normal_gradient(n, 5e-4, seed=442)
    i1, v1, s1, r1, _ = gpu_compress(g, r0, [10.0])
    l2 = check_recompress(i1, v1, 10.0, residual=r1, what="level 2")
    l3 = check_recompress(l2[0], l2[1], 10.0, residual=l2[3], what="level 3")
    di, dv, ds, dr = oracle_compress(g, r0, [1000.0])
    assert np.array_equal(l3[0], di) and np.array_equal(l3[1].view(np.uint32), dv.view(np.uint32))
    assert np.array_equal(l3[3].view(np.uint32), dr.view(np.uint32))
    np.testing.assert_allclose(s1[0, 0, 2] * l2[2][0, 2] * l3[2][0, 2], ds[0, 0, 2], rtol=STAT_RTOL)


def test_recompress_argument_checks():
    k1 = 1000
    idx1 = torch.arange(k1, dtype=torch.int32, device="cuda")
    val1 = torch.ones(k1, dtype=torch.float32, device="cuda")
    ws = torch.empty(binding.gravac_workspace_bytes(k1, 1, 0), dtype=torch.uint8, device="cuda")
    oi = torch.empty(100, dtype=torch.int32, device="cuda")
    ov = torch.empty(100, dtype=torch.float32, device="cuda")
    st = torch.zeros(1, 4, dtype=torch.float64, device="cuda")
    kw = dict(out_idx=oi, out_val=ov, out_stats=st, workspace=ws)
    with pytest.raises(binding.GravacError) as e:
        binding.gravac_recompress(idx1, val1, 0.5, **kw)
    assert e.value.code == binding.ERR_INVALID_ARG
    with pytest.raises(binding.GravacError) as e:
        binding.gravac_recompress(idx1, val1, 2.0, **kw)          # k2 = 500 > capacity 100
    assert e.value.code == binding.ERR_CAPACITY
    with pytest.raises(binding.GravacError) as e:
        binding.gravac_recompress(idx1, val1, 10.0, seg_counts=[400, 500], **kw)   # counts do not add up to k1
    assert e.value.code == binding.ERR_INVALID_ARG
    with pytest.raises(binding.GravacError) as e:
        binding.gravac_recompress(idx1, val1, 10.0, seg_counts=[1000, 0], **kw)
    assert e.value.code == binding.ERR_INVALID_ARG
    with pytest.raises(binding.GravacError) as e:
        binding.gravac_recompress(idx1, val1, 10.0, out_idx=oi, out_val=ov, out_stats=st, workspace=ws[:4096])
    assert e.value.code == binding.ERR_WORKSPACE
    torch.cuda.synchronize()
