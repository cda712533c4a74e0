"""GPU parity of Random-k with error feedback: gravac_randomk_compress against the CPU oracle, element by
element through the C ABI.  Indices, values, residuals and the threshold priority bit-exact; sums within
1e-5 relative."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2305_12201_amd import binding, workloads
from tests.gpu_util import assert_same

pytestmark = pytest.mark.gpu

FB = binding.FLAG_FORCE_FALLBACK


def gpu_randomk(grad, residual, cfs, seed, commit=0, seg=None, flags=0, comp=None):
    n = grad.size
    g = torch.from_numpy(grad).cuda()
    r = torch.from_numpy(residual.copy()).cuda()
    if comp is None:
        comp = binding.Compressor(n, cfs, commit, seg)
    comp.out_idx.fill_(-1)
    comp.out_val.fill_(float("nan"))
    idx, val, stats = comp.randomk(g, r, seed, flags=flags)
    torch.cuda.synchronize()
    st = comp.status()
    assert st["internal_error"] == 0
    assert int(comp.out_count.item()) == comp.k_total
    assert np.array_equal(g.cpu().numpy().view(np.uint32), grad.view(np.uint32)), "gradient modified"
    return idx.cpu().numpy(), val.cpu().numpy(), stats.cpu().numpy(), r.cpu().numpy(), st


def check(grad, residual, cfs, seed, commit=0, seg=None, flags=0, what=""):
    gpu = gpu_randomk(grad, residual, cfs, seed, commit, seg, flags)
    res = residual.copy()
    idx, val, stats = oracle.randomk_compress(grad, res, cfs, seed, commit, seg)
    assert_same(gpu, (idx, val, stats, res), what)
    return gpu


@pytest.mark.parametrize("n", [1, 2, 3, 63, 64, 65, 1023, 1025, 4097, 8191, 8192, 8193, 16_385, 100_003, 1_048_576,
                               3_000_001])
def test_ragged_sizes(n):
    g = workloads.normal_gradient(n, 1e-3, seed=n)
    r = workloads.normal_gradient(n, 1e-4, seed=n + 1)
    for cf in (1.0, 2.5, 100.0):
        check(g, r, [cf], seed=n * 7 + int(cf), what=f"n={n} cf={cf}")


@pytest.mark.parametrize("flags", [0, FB])
def test_multi_cf_every_commit_and_seeds(flags):
    n = 1_500_007
    g = workloads.resnet_like_gradient(n, seed=11)
    r = workloads.normal_gradient(n, 1e-5, seed=12)
    cfs = [10.0, 100.0, 1000.0]
    sel = []
    for commit in range(3):
        gpu = check(g, r, cfs, seed=2 ** 40 + 5, commit=commit, flags=flags, what=f"commit {commit}")
        assert bool(gpu[4]["any_fallback"]) == bool(flags)
        sel.append(set(gpu[0].tolist()))
    assert sel[2] < sel[1] < sel[0]
    other = check(g, r, cfs, seed=2 ** 40 + 6, commit=1, flags=flags, what="another seed")
    assert set(other[0].tolist()) != sel[1]
    # the values do not influence the draw
    same = check(-g * np.float32(3), r, cfs, seed=2 ** 40 + 5, commit=1, flags=flags, what="other values")
    assert set(same[0].tolist()) == sel[1]


@pytest.mark.parametrize("flags", [0, FB])
def test_layerwise(flags):
    sizes = [64, 1, 4096, 37, 100_003, 2, 9408, 64, 64, 1000, 4097, 8191, 3, 250_001, 5, 700_000]
    off = workloads.offsets_of(sizes)
    n = int(off[-1])
    g = workloads.resnet_like_gradient(n, seed=21)
    r = workloads.normal_gradient(n, 1e-5, seed=22)
    seg = check(g, r, [100.0], seed=99, seg=off, flags=flags, what="layerwise cf100")
    check(g, r, [10.0, 100.0], seed=99, commit=0, seg=off, flags=flags, what="layerwise two CFs")
    assert seg[2].shape == (len(sizes), 1, 4)


def test_resnet_tensor_list_reduced_and_iterations():
    sizes = workloads.scaled_sizes(workloads.resnet101_tensor_sizes(), 16)
    off = workloads.offsets_of(sizes)
    n = int(off[-1])
    comp = binding.Compressor(n, [100.0], 0, off)
    res_gpu = np.zeros(n, np.float32)
    res_ref = np.zeros(n, np.float32)
    for it in range(4):
        g = workloads.config5_worker_grad(it, n)
        gpu = gpu_randomk(g, res_gpu, [100.0], seed=it, seg=off, comp=comp)
        idx, val, stats = oracle.randomk_compress(g, res_ref, [100.0], it, 0, off)
        assert_same(gpu, (idx, val, stats, res_ref), f"iteration {it}")
        res_gpu = gpu[3]


def test_specials_and_constant_input():
    n = 200_000
    g = np.ones(n, np.float32)
    gpu = check(g, np.zeros(n, np.float32), [10.0], seed=1, what="ones")
    assert gpu[2][0, 0, 2] == pytest.approx(0.1, rel=1e-12)
    g = workloads.normal_gradient(n, 1e-3, seed=31)
    g[::1000] = np.inf
    g[1::1000] = -0.0
    g[2::1000] = 1e-42
    gpu = gpu_randomk(g, np.zeros(n, np.float32), [4.0], seed=3)
    res = np.zeros(n, np.float32)
    idx, val, stats = oracle.randomk_compress(g, res, [4.0], 3)
    assert np.array_equal(gpu[0], idx) and np.array_equal(gpu[1].view(np.uint32), val.view(np.uint32))
    assert np.array_equal(gpu[3].view(np.uint32), res.view(np.uint32))
    assert gpu[2][0, 0, 3] == stats[0, 0, 3]


@pytest.mark.fullsize
def test_full_size_resnet101():
    n = workloads.RESNET101_N
    g = workloads.config2_grad(0)
    r = workloads.config2_residual0()
    check(g, r, [10.0, 100.0, 1000.0], seed=2024, commit=1, what="44.5M elements")
