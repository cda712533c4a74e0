"""Seeded random cases through every mode of the compression call (flat and layerwise, one to four CFs, any
commit position, sampled bounds, forced exact route, carried residuals on one workspace, Top-k and
Random-k), each compared with the CPU oracle element by element.  The cases are drawn from a fixed seed, so
the test is the same on every run."""
import os

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2305_12201_amd import binding
from tests.gpu_util import STAT_RTOL, assert_same, gpu_compress, oracle_compress

pytestmark = pytest.mark.gpu

# number of cases of every sweep; GRAVAC_RANDOM_CASES widens the sweeps for a longer run
N_CASES = int(os.environ.get("GRAVAC_RANDOM_CASES", "0"))

CF_POOL = [1.0, 1.5, 2.0, 7.0, 10.0, 33.3, 100.0, 1000.0, 12345.0]


def _values(rng, n):
    """One of several value families: heavy tails, exact zeros, few distinct values (ties), a knee, huge range."""
    kind = rng.integers(0, 6)
    if kind == 0:
        x = rng.standard_normal(n) * 1e-3
    elif kind == 1:
        x = rng.laplace(0.0, 1e-4, n)
        m = rng.random(n) < 0.01
        x[m] *= 100.0
    elif kind == 2:
        x = rng.standard_normal(n) * 1e-4
        x[rng.random(n) < rng.choice([0.5, 0.95])] = 0.0
    elif kind == 3:
        x = rng.integers(-5, 6, n) * 0.25
    elif kind == 4:
        x = rng.standard_normal(n) * 1e-6
        m = rng.random(n) < 0.02
        x[m] = np.exp(rng.uniform(-3.0, 8.0, int(m.sum()))) * rng.choice([-1.0, 1.0], int(m.sum()))
    else:
        x = rng.standard_normal(n) * np.exp(rng.uniform(-20.0, 20.0, n))
    return x.astype(np.float32)


def _segments(rng, n):
    if n < 4 or rng.random() < 0.5:
        return None
    parts = int(min(n, rng.integers(2, 25)))
    cuts = np.sort(rng.choice(np.arange(1, n), parts - 1, replace=False))
    return np.concatenate([[0], cuts, [n]]).astype(np.int64)


@pytest.mark.parametrize("case", range(N_CASES or 120))
def test_random_case(case):
    rng = np.random.Generator(np.random.PCG64(1000 + case))
    n = int(rng.choice([rng.integers(1, 300), rng.integers(300, 20_000), rng.integers(20_000, 400_000)]))
    n_cf = int(rng.integers(1, 5))
    cfs = sorted(float(c) for c in rng.choice(CF_POOL, n_cf, replace=False))
    commit = int(rng.integers(0, n_cf))
    seg = _segments(rng, n)
    what = f"case {case}: n={n} cfs={cfs} commit={commit} segments={0 if seg is None else seg.size - 1}"
    comp = binding.Compressor(n, cfs, commit, seg)
    res_gpu = _values(rng, n) * np.float32(0.1)
    res_ref = res_gpu.copy()
    flags_seq = [int(rng.choice([0, binding.FLAG_FORCE_FALLBACK])), 0, int(rng.choice([0, binding.FLAG_FORCE_FALLBACK]))]
    for it, flags in enumerate(flags_seq):
        g = _values(rng, n)
        gpu = gpu_compress(g, res_gpu, cfs, commit, seg, flags=flags, comp=comp)
        ref = oracle_compress(g, res_ref, cfs, commit, seg)
        assert gpu[4]["internal_error"] == 0, what
        assert_same(gpu, ref, f"{what} iteration {it} flags {flags}")
        res_gpu, res_ref = gpu[3], ref[3]
    # the same shape through Random-k (one call, residual from above)
    g = _values(rng, n)
    seed = int(rng.integers(0, 2**63))
    gt, rt = torch.from_numpy(g).cuda(), torch.from_numpy(res_gpu.copy()).cuda()
    idx, val, stats = comp.randomk(gt, rt, seed)
    torch.cuda.synchronize()
    assert comp.status()["internal_error"] == 0, what
    ref_res = res_ref.copy()
    ri, rv, rs = oracle.randomk_compress(g, ref_res, cfs, seed, commit, seg)
    assert np.array_equal(idx.cpu().numpy(), ri), f"{what}: Random-k indices"
    assert np.array_equal(val.cpu().numpy().view(np.uint32), rv.view(np.uint32)), f"{what}: Random-k values"
    assert np.array_equal(rt.cpu().numpy().view(np.uint32), ref_res.view(np.uint32)), f"{what}: Random-k residual"
    np.testing.assert_allclose(stats.cpu().numpy()[..., :3], rs[..., :3], rtol=STAT_RTOL, atol=0, equal_nan=True, err_msg=what)


@pytest.mark.parametrize("case", range(N_CASES or 40))
def test_random_decompress(case):
    """W index-sorted messages of random lengths (some empty, some dense, some thin, some in one cluster) into a
    dense buffer that already holds values, with and without the workspace; every third case as the parameter
    update with a multiplier.  In half of the cases every message is thin, so that whole stretches of the buffer
    are named by a few pairs only."""
    rng = np.random.Generator(np.random.PCG64(5000 + case))
    n = int(rng.choice([rng.integers(1, 9000), rng.integers(9000, 600_000), rng.integers(600_000, 3_000_000)]))
    W = int(rng.choice([1, 2, 8, 8, 17, 64, 70]))
    thin_only = rng.random() < 0.5
    alpha = None if case % 3 else float(rng.choice([-0.0125, 0.3, -2.5, 1.0]))
    idx, val, ks = [], [], []
    for w in range(W):
        mode = int(rng.choice([0, 3, 4, 4])) if thin_only else int(rng.integers(0, 5))
        if mode == 0:
            k = 0
        elif mode == 1:
            k = int(rng.integers(1, n + 1)) if n < 600_000 else int(rng.integers(1, n // 8))
        elif mode == 4:
            k = int(rng.integers(1, max(2, n // (250 * W) + 1)))      # about 30 pairs of all workers per 8192 entries
        else:
            k = int(rng.integers(1, max(2, n // 50 + 1)))
        if thin_only and mode == 3:
            k = min(k, 200)
        if mode == 3 and n > 10:                       # all pairs inside one short range
            lo = int(rng.integers(0, n - min(n, 4 * k) + 1))
            pos = lo + np.sort(rng.choice(min(n - lo, 4 * k), min(k, min(n - lo, 4 * k)), replace=False))
        else:
            pos = np.sort(rng.choice(n, k, replace=False))
        idx.append(pos.astype(np.int32))
        val.append((rng.standard_normal(pos.size) * 1e-2).astype(np.float32))
        ks.append(int(pos.size))
    if W > 1 and ks[0] and ks[1]:                      # some entries named by the first two workers alike
        m = min(ks[0], ks[1], 50)
        take = np.sort(rng.choice(ks[0], m, replace=False))
        idx[1] = np.union1d(idx[1], idx[0][take]).astype(np.int32)
        val[1] = (rng.standard_normal(idx[1].size) * 1e-2).astype(np.float32)
        ks[1] = int(idx[1].size)
    idx = np.concatenate(idx) if sum(ks) else np.zeros(0, np.int32)
    val = np.concatenate(val) if sum(ks) else np.zeros(0, np.float32)
    base = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    want = base.copy()
    if alpha is None:
        oracle.decompress_accumulate(idx, val, ks, want)
    else:
        oracle.decompress_update(idx, val, ks, alpha, want)
    ti = torch.from_numpy(idx).cuda() if idx.size else torch.zeros(1, dtype=torch.int32, device="cuda")
    tv = torch.from_numpy(val).cuda() if val.size else torch.zeros(1, dtype=torch.float32, device="cuda")
    for ws in (None, torch.empty(binding.gravac_decompress_workspace_bytes(W, n), dtype=torch.uint8, device="cuda")):
        d = torch.from_numpy(base.copy()).cuda()
        if alpha is None:
            binding.gravac_decompress_accumulate(ti, tv, ks, d, workspace=ws)
        else:
            binding.gravac_decompress_update(ti, tv, ks, alpha, d, workspace=ws)
        torch.cuda.synchronize()
        got = d.cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), \
            f"case {case}: n={n} W={W} alpha={alpha} workspace={ws is not None}: differs at {np.nonzero(got != want)[0][:5]}"


@pytest.mark.parametrize("case", range(N_CASES or 30))
def test_random_two_levels(case):
    """Level 1 at a random CF, then the second-level Top-k on its message with deferred commit: message, statistics
    and the residual it leaves, against the oracle's two-level path."""
    rng = np.random.Generator(np.random.PCG64(9000 + case))
    n = int(rng.choice([rng.integers(50, 3000), rng.integers(3000, 300_000)]))
    cf1 = float(rng.choice([2.0, 5.0, 10.0, 40.0]))
    cf_rel = float(rng.choice([1.0, 1.5, 2.0, 4.0, 10.0, 100.0]))
    seg = _segments(rng, n)
    g, r0 = _values(rng, n), _values(rng, n) * np.float32(0.1)
    comp = binding.Compressor(n, [cf1], 0, seg)
    gt, rt = torch.from_numpy(g).cuda(), torch.from_numpy(r0.copy()).cuda()
    i1, v1, _ = comp(gt, rt)
    torch.cuda.synchronize()
    ref_res = r0.copy()
    ri1, rv1, _ = oracle.compress(g, ref_res, [cf1], 0, seg)
    assert np.array_equal(i1.cpu().numpy(), ri1)
    sizes = [n] if seg is None else np.diff(seg).tolist()
    counts = None if seg is None else [binding.gravac_topk_count(int(s), cf1) for s in sizes]
    k1 = int(i1.numel())
    k2 = binding.gravac_topk_count(k1, cf_rel) if counts is None else sum(binding.gravac_topk_count(c, cf_rel) for c in counts)
    rows = 1 if counts is None else len(counts)
    oi = torch.empty(k2, dtype=torch.int32, device="cuda")
    ov = torch.empty(k2, dtype=torch.float32, device="cuda")
    st = torch.zeros(rows, 4, dtype=torch.float64, device="cuda")
    ws = torch.empty(binding.gravac_workspace_bytes(k1, 1, 0 if counts is None else len(counts)), dtype=torch.uint8, device="cuda")
    binding.gravac_recompress(i1, v1, cf_rel, counts, rt, out_idx=oi, out_val=ov, out_stats=st, workspace=ws)
    torch.cuda.synchronize()
    assert binding.gravac_read_status(ws)["internal_error"] == 0
    ri2, rv2, rs2 = oracle.recompress(ri1, rv1, cf_rel, ref_res, counts)
    what = f"case {case}: n={n} cf1={cf1} cf_rel={cf_rel} segments={rows}"
    assert np.array_equal(oi.cpu().numpy(), ri2), what
    assert np.array_equal(ov.cpu().numpy().view(np.uint32), rv2.view(np.uint32)), what
    assert np.array_equal(rt.cpu().numpy().view(np.uint32), ref_res.view(np.uint32)), what
    np.testing.assert_allclose(st.cpu().numpy()[..., :3], rs2[..., :3], rtol=STAT_RTOL, atol=0, equal_nan=True, err_msg=what)
