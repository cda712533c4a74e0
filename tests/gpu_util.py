"""Helpers shared by the GPU parity tests: run the HIP library and the CPU oracle on the same inputs."""
import numpy as np
import torch

from oracle import oracle
from paper_2305_12201_amd import binding

STAT_RTOL = 1e-5   # tolerance on the statistics (fp64 sums in a different order); everything else is bit-exact


def gpu_compress(grad, residual, cfs, commit=0, seg=None, flags=0, comp=None):
    """Run gravac_compress on host arrays; returns (idx, val, stats, new_residual, status) as numpy."""
    n = grad.size
    g = torch.from_numpy(grad).cuda()
    r = torch.from_numpy(residual.copy()).cuda()
    if comp is None:
        comp = binding.Compressor(n, cfs, commit, seg)
    comp.out_idx.fill_(-1)
    comp.out_val.fill_(float("nan"))
    idx, val, stats = comp(g, r, flags=flags)
    torch.cuda.synchronize()
    st = comp.status()
    assert int(comp.out_count.item()) == comp.k_total
    return idx.cpu().numpy(), val.cpu().numpy(), stats.cpu().numpy(), r.cpu().numpy(), st


def assert_same(gpu, ref, what=""):
    """gpu = (idx, val, stats, res[, status]); ref = (idx, val, stats, res) from the oracle."""
    gi, gv, gs, gr = gpu[:4]
    oi, ov, os_, or_ = ref
    assert gi.shape == oi.shape, what
    assert np.array_equal(gi, oi), f"{what}: indices differ at {np.nonzero(gi != oi)[0][:5]}"
    assert np.array_equal(gv.view(np.uint32), ov.view(np.uint32)), f"{what}: values differ"
    assert np.array_equal(gr.view(np.uint32), or_.view(np.uint32)), \
        f"{what}: residual differs at {np.nonzero(gr.view(np.uint32) != or_.view(np.uint32))[0][:5]}"
    assert gs.shape == os_.shape
    # tau is exact; sums agree to rounding order
    assert np.array_equal(gs[..., 3], os_[..., 3], equal_nan=True), f"{what}: thresholds differ"
    np.testing.assert_allclose(gs[..., :3], os_[..., :3], rtol=STAT_RTOL, atol=0, equal_nan=True, err_msg=what)


def oracle_compress(grad, residual, cfs, commit=0, seg=None):
    res = residual.copy()
    idx, val, stats = oracle.compress(grad, res, cfs, commit, seg)
    return idx, val, stats, res


def check(grad, residual, cfs, commit=0, seg=None, flags=0, what="", expect_fallback=None):
    gpu = gpu_compress(grad, residual, cfs, commit, seg, flags)
    ref = oracle_compress(grad, residual, cfs, commit, seg)
    assert gpu[4]["internal_error"] == 0, f"{what}: internal error flag set"
    assert_same(gpu, ref, what)
    if expect_fallback is not None:
        assert bool(gpu[4]["any_fallback"]) == expect_fallback, f"{what}: fallback={gpu[4]}"
    return gpu, ref
