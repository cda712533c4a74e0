"""GPU parity of the threshold sparsifier (gravac_threshold_compress) against the oracle, through the C ABI:
indices, values and residual bit for bit, the count exactly, statistics within 1e-5 relative."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2305_12201_amd import binding, workloads
from tests.gpu_util import STAT_RTOL

pytestmark = pytest.mark.gpu


def run(grad, residual, tau, capacity=None, ws=None):
    n = grad.size
    cap = n if capacity is None else capacity
    g = torch.from_numpy(grad).cuda()
    r = torch.from_numpy(residual.copy()).cuda()
    oi = torch.full((max(cap, 1),), -1, dtype=torch.int32, device="cuda")[:cap]
    ov = torch.full((max(cap, 1),), float("nan"), dtype=torch.float32, device="cuda")[:cap]
    cnt = torch.full((1,), -7, dtype=torch.int64, device="cuda")
    st = torch.zeros(4, dtype=torch.float64, device="cuda")
    if ws is None:
        ws = torch.empty(binding.gravac_workspace_bytes(n, 1, 0), dtype=torch.uint8, device="cuda")
    binding.gravac_threshold_compress(g, r, tau, out_idx=oi, out_val=ov, out_count=cnt, out_stats=st, workspace=ws)
    torch.cuda.synchronize()
    assert binding.gravac_read_status(ws)["internal_error"] == 0
    c = int(cnt.item())
    return oi.cpu().numpy(), ov.cpu().numpy(), st.cpu().numpy(), r.cpu().numpy(), c


def check(grad, residual, tau, capacity=None, what=""):
    oi, ov, st, res, c = run(grad, residual, tau, capacity)
    ref_res = residual.copy()
    ri, rv, rs, rc = oracle.threshold_compress(grad, ref_res, tau, capacity)
    assert c == rc, what
    k = ri.size                                     # 0 if the selection does not fit
    assert np.array_equal(oi[:k], ri), what
    assert np.array_equal(ov[:k].view(np.uint32), rv.view(np.uint32)), what
    assert np.all(oi[k:] == -1), f"{what}: written past the message"
    assert np.array_equal(res.view(np.uint32), ref_res.view(np.uint32)), \
        f"{what}: residual differs at {np.nonzero(res.view(np.uint32) != ref_res.view(np.uint32))[0][:5]}"
    assert st[3] == rs[3], what
    np.testing.assert_allclose(st[:3], rs[:3], rtol=STAT_RTOL, atol=0, err_msg=what)
    return c


@pytest.mark.parametrize("n", [1, 5, 64, 1023, 4097, 8192, 8193, 100_003, 300_001])
def test_ragged_sizes_and_every_regime(n):
    g = workloads.normal_gradient(n, 1e-3, seed=n)
    r = workloads.normal_gradient(n, 1e-4, seed=n + 1)
    for tau in (1e-9, 3e-4, 1e-3, 3e-3, 1.0):       # everything kept ... nothing kept
        check(g, r, tau, what=f"n={n} tau={tau}")


def test_ties_at_tau_signed_zeros_denormals_and_specials():
    rng = np.random.default_rng(3)
    n = 70_000
    g = (rng.integers(-6, 7, n) * 0.125).astype(np.float32)
    r = (rng.integers(-2, 3, n) * 0.125).astype(np.float32)
    g[rng.random(n) < 0.1] = -0.0
    for tau in (0.125, 0.25, 0.5, 1.0):             # thousands of entries equal to tau: all kept
        check(g, r, tau, what=f"ties tau={tau}")
    d = (rng.integers(-50, 51, 5000).astype(np.float32) * np.float32(1e-41))
    check(d, np.zeros(5000, np.float32), 2e-40, what="denormals")
    s = workloads.normal_gradient(10_000, 1.0, seed=9)
    s[[5, 77, 9000]] = [np.inf, -np.inf, np.nan]
    oi, ov, st, res, c = run(s, np.zeros(10_000, np.float32), 2.5)
    ref_res = np.zeros(10_000, np.float32)
    ri, rv, rs, rc = oracle.threshold_compress(s, ref_res, 2.5)
    assert c == rc and np.array_equal(oi[:c], ri) and {5, 77, 9000} <= set(ri.tolist())
    assert np.array_equal(ov[:c].view(np.uint32), rv.view(np.uint32))
    assert np.array_equal(res.view(np.uint32), ref_res.view(np.uint32))


def test_dense_and_sparse_sub_tiles_iterations_and_workspace_shared_with_topk():
    n_conv, n_fc = 301_111, 2_000_003
    n = n_conv + n_fc
    ws = torch.empty(binding.gravac_workspace_bytes(n, 1, 0), dtype=torch.uint8, device="cuda")
    comp = binding.Compressor(n, [100.0], 0)
    comp.workspace = ws
    res_gpu = np.zeros(n, np.float32)
    res_ref = np.zeros(n, np.float32)
    for it in range(3):
        g = workloads.config3_grad(it, n_conv, n_fc)          # conv part: most entries above 1e-4, fc part: few
        oi, ov, st, new_res, c = run(g, res_gpu, 1e-4, ws=ws)
        ri, rv, rs, rc = oracle.threshold_compress(g, res_ref, 1e-4)
        assert c == rc and np.array_equal(oi[:c], ri) and np.array_equal(ov[:c].view(np.uint32), rv.view(np.uint32))
        assert np.array_equal(new_res.view(np.uint32), res_ref.view(np.uint32)), f"iteration {it}"
        np.testing.assert_allclose(st[:3], rs[:3], rtol=STAT_RTOL)
        res_gpu = new_res
        # a Top-k call on the same workspace in between: neither disturbs the other
        gt, rt = torch.from_numpy(g).cuda(), torch.zeros(n, dtype=torch.float32, device="cuda")
        comp(gt, rt)
        torch.cuda.synchronize()
        assert comp.status()["internal_error"] == 0


def test_capacity_too_small_emits_nothing_and_removes_nothing():
    n = 500_000
    g = workloads.resnet_like_gradient(n, seed=4)
    r = workloads.normal_gradient(n, 1e-5, seed=5)
    c = check(g, r, 3e-4, what="fits")
    assert c > 1000
    for cap in (c, c - 1, c // 2, 0):
        assert check(g, r, 3e-4, capacity=cap, what=f"capacity {cap}") == c
    # dense selection (sub-tiles without a candidate list) that does not fit
    assert check(g, r, 1e-7, capacity=1000, what="dense, too small") > n // 2


def test_equals_topk_at_its_own_threshold():
    n = 1_200_003
    g = workloads.normal_gradient(n, 1e-3, seed=21)
    r = np.zeros(n, np.float32)
    comp = binding.Compressor(n, [100.0], 0)
    gt, rt = torch.from_numpy(g).cuda(), torch.from_numpy(r).cuda()
    idx, val, stats = comp(gt, rt)
    torch.cuda.synchronize()
    tau = float(stats[0, 0, 3])
    oi, ov, st, res, c = run(g, r, tau)
    assert c == comp.k_total and np.array_equal(oi[:c], idx.cpu().numpy())
    assert np.array_equal(res.view(np.uint32), rt.cpu().numpy().view(np.uint32))


def test_full_size_resnet101_shape():
    n = workloads.RESNET101_N
    g = workloads.config2_grad(0)
    r = workloads.config2_residual0()
    check(g, r, 5e-4, what="ResNet101 shape")


def test_bad_arguments():
    n = 1000
    g = torch.zeros(n, device="cuda"); r = torch.zeros(n, device="cuda")
    oi = torch.zeros(10, dtype=torch.int32, device="cuda"); ov = torch.zeros(10, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda"); st = torch.zeros(4, dtype=torch.float64, device="cuda")
    ws = torch.empty(binding.gravac_workspace_bytes(n, 1, 0), dtype=torch.uint8, device="cuda")
    for tau in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(binding.GravacError) as e:
            binding.gravac_threshold_compress(g, r, tau, out_idx=oi, out_val=ov, out_count=cnt, out_stats=st, workspace=ws)
        assert e.value.code == binding.ERR_INVALID_ARG
    with pytest.raises(binding.GravacError) as e:
        binding.gravac_threshold_compress(g, r, 1.0, out_idx=oi, out_val=ov, out_count=cnt, out_stats=st,
                                          workspace=ws[:256])
    assert e.value.code == binding.ERR_WORKSPACE
    torch.cuda.synchronize()
