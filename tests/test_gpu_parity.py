"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI.

Bit-exact on indices, values and residuals; statistics within 1e-5 relative (fp64 sums in a
different order); the threshold magnitude exactly.  Sizes are chosen so the full-sort oracle
finishes in seconds while the GPU path still spans many wave tiles and a ragged tail.
"""
import numpy as np
import pytest
import torch

from paper_2305_12201_amd import binding, workloads
from tests.gpu_util import assert_same, check, gpu_compress, oracle_compress

pytestmark = pytest.mark.gpu

FB = binding.FLAG_FORCE_FALLBACK


def test_library_is_loaded_from_the_tree():
    import os
    assert os.path.exists(binding.library_path())
    assert binding.lib() is not None


# --------------------------------------------------------------------------
# configuration 1: N = 2^20, Normal(0, 1e-3), CF 100, two iterations carrying the residual
# --------------------------------------------------------------------------

@pytest.mark.parametrize("flags", [0, FB])
def test_config1_two_iterations(flags):
    n = 1 << 20
    res_gpu = np.zeros(n, np.float32)
    res_ref = np.zeros(n, np.float32)
    for it in range(2):
        g = workloads.config1(it)
        gpu = gpu_compress(g, res_gpu, [100.0], flags=flags)
        ref = oracle_compress(g, res_ref, [100.0])
        assert gpu[0].size == 10486
        assert_same(gpu, ref, f"config1 it{it}")
        assert gpu[4]["internal_error"] == 0
        assert bool(gpu[4]["any_fallback"]) == bool(flags)
        res_gpu, res_ref = gpu[3], ref[3]


# --------------------------------------------------------------------------
# ragged sizes, tiny inputs, every CF regime
# --------------------------------------------------------------------------

@pytest.mark.parametrize("n", [1, 2, 3, 5, 63, 64, 65, 255, 257, 1023, 1025, 4095, 4096, 4097, 8191, 8192, 8193,
                               16_385, 100_003, 131_072, 131_073, 300_001])
def test_ragged_sizes(n):
    g = workloads.normal_gradient(n, 1e-3, seed=n)
    r = workloads.normal_gradient(n, 1e-4, seed=n + 1)
    for cf in (1.0, 1.5, 10.0, 1000.0):
        check(g, r, [cf], what=f"n={n} cf={cf}")
    check(g, r, [3.0], flags=FB, what=f"n={n} forced", expect_fallback=True)


def test_heavy_ties_and_signed_zeros():
    rng = np.random.default_rng(7)
    for n in (1000, 70_000, 500_000):
        g = (rng.integers(-6, 7, n) * 0.125).astype(np.float32)
        r = (rng.integers(-2, 3, n) * 0.125).astype(np.float32)
        g[rng.random(n) < 0.1] = -0.0
        for cf in (2.0, 7.0, 100.0):
            check(g, r, [cf], what=f"ties n={n} cf={cf}")
            check(g, r, [cf], flags=FB, what=f"ties forced n={n} cf={cf}")


def test_all_zero_and_all_equal():
    n = 50_000
    z = np.zeros(n, np.float32)
    gpu, ref = check(z, z, [10.0], what="all zero")
    assert gpu[2][0, 0].tolist() == [0.0, 0.0, 1.0, 0.0]
    one = np.full(n, -0.5, np.float32)
    check(one, z, [100.0], what="all equal")
    check(one, z, [100.0], flags=FB, what="all equal forced")


def test_k_exceeds_nonzeros():
    n = 200_000
    g = np.zeros(n, np.float32)
    rng = np.random.default_rng(3)
    pos = rng.choice(n, 500, replace=False)
    g[pos] = rng.standard_normal(500).astype(np.float32)
    check(g, np.zeros(n, np.float32), [100.0], what="k=2000 > 500 nonzeros")


def test_nan_inf_and_denormals():
    n = 10_000
    g = workloads.normal_gradient(n, 1e-3, seed=5)
    g[17] = np.inf
    g[99] = -np.inf
    g[5000] = np.nan
    g[6000:6100] = 1e-40
    check(g, np.zeros(n, np.float32), [100.0], what="nan/inf")
    d = np.full(n, 1e-40, np.float32)
    d[::7] = -3e-41
    gpu, ref = check(d, d.copy(), [10.0], what="denormals")
    assert np.all(gpu[1] != 0)          # denormal sums are not flushed


def test_extreme_dynamic_range_and_outliers():
    n = 400_000
    rng = np.random.default_rng(11)
    g = (rng.standard_normal(n) * np.exp(rng.uniform(-30, 30, n))).astype(np.float32)
    check(g, np.zeros(n, np.float32), [10.0, 100.0, 1000.0], commit=1, what="wide range")
    # a sample cannot see a handful of huge entries: the bound is too low, never too high
    g = workloads.normal_gradient(n, 1e-6, seed=2)
    g[rng.choice(n, 37, replace=False)] = 5.0
    check(g, np.zeros(n, np.float32), [1000.0, 10000.0], commit=0, what="rare outliers")


def test_clustered_top_entries_hidden_from_the_sample():
    # all large entries sit in one short run: a strided sample underestimates the tail and the
    # library must notice (fewer candidates than k) and take the exact route
    n = 1_000_000
    g = workloads.normal_gradient(n, 1e-6, seed=9)
    g[123_456:123_456 + 3000] = workloads.normal_gradient(3000, 1.0, seed=10)
    gpu, ref = check(g, np.zeros(n, np.float32), [100.0], what="clustered")
    assert gpu[4]["internal_error"] == 0


def _knee_gradient(n, seed):
    """A tiny body, 12,500 large entries spread over seven octaves, and between them a cluster of 5000 entries
    within 4096 neighbouring bit patterns.  At CF 100 (k = n / 100 = 15,000) the k-th largest lies inside the
    cluster, while the sampled ranks that bracket it fall into the body and into the large entries: the bracket is
    many octaves wide, so the histogram bin that holds the k-th largest is coarse and holds the whole cluster."""
    rng = np.random.Generator(np.random.PCG64(seed))
    g = workloads.normal_gradient(n, 1e-6, seed=seed + 1)
    pos = rng.permutation(n)[:17_500]
    big = np.exp(rng.uniform(np.log(50.0), np.log(5000.0), 12_500)) * rng.choice([-1.0, 1.0], 12_500)
    g[pos[:12_500]] = big.astype(np.float32)
    bits = np.float32(1.0).view(np.uint32) + rng.integers(0, 4096, 5000, dtype=np.uint32)
    g[pos[12_500:]] = bits.view(np.float32) * rng.choice([-1.0, 1.0], 5000).astype(np.float32)
    return g


def test_full_coarse_bin_is_binned_again_inside_the_bin():
    # the located bin is more than 2^11 keys wide and holds more keys than a gather list: the CF concerned is
    # binned again inside that bin (no second pass over the gradient), the other CF keeps its plan
    n = 1_500_000
    g = _knee_gradient(n, seed=71)
    for cfs, commit in (([100.0], 0), ([100.0, 1000.0], 0), ([100.0, 1000.0], 1), ([10.0, 100.0, 1000.0], 1)):
        gpu, ref = check(g, np.zeros(n, np.float32), cfs, commit=commit, what=f"knee cfs={cfs} commit={commit}",
                         expect_fallback=True)
        assert gpu[4]["narrow_fallback_segments"] == 1, gpu[4]
    # layerwise: only the middle tensor has the knee
    parts = [workloads.normal_gradient(300_001, 1e-3, seed=72), g, workloads.resnet_like_gradient(200_003, seed=73)]
    flat = np.concatenate(parts)
    seg = np.cumsum([0] + [x.size for x in parts]).astype(np.int64)
    gpu, ref = check(flat, np.zeros(flat.size, np.float32), [100.0, 1000.0], commit=0, seg=seg, what="knee, layerwise",
                     expect_fallback=True)
    assert gpu[4]["fallback_segments"] == 1 and gpu[4]["narrow_fallback_segments"] == 1, gpu[4]
    # more iterations on the same workspace (what the narrow route left there is what the next call finds)
    comp = binding.Compressor(n, [100.0, 1000.0], 0)
    r = np.zeros(n, np.float32)
    for it in range(3):
        gpu = gpu_compress(g, r, [100.0, 1000.0], 0, comp=comp)
        ref = oracle_compress(g, r, [100.0, 1000.0], 0)
        assert gpu[4]["internal_error"] == 0
        assert_same(gpu, ref, f"knee, iteration {it}")
        r = ref[3]


# --------------------------------------------------------------------------
# several CFs in one call, every commit position
# --------------------------------------------------------------------------

@pytest.mark.parametrize("flags", [0, FB])
def test_multi_cf_every_commit(flags):
    n = 700_001
    g = workloads.resnet_like_gradient(n, seed=21)
    r = workloads.normal_gradient(n, 1e-5, seed=22)
    cfs = [10.0, 100.0, 1000.0]
    for commit in range(3):
        check(g, r, cfs, commit=commit, flags=flags, what=f"commit={commit}")
    check(g, r, [1.5, 2.0, 3.0, 10.0, 50.0, 100.0, 1000.0, 5000.0], commit=5, flags=flags, what="8 CFs")


# --------------------------------------------------------------------------
# reduced twins of configurations 2-4, residual carried over iterations
# --------------------------------------------------------------------------

def test_config2_reduced_five_iterations():
    n = 2_000_003
    res_gpu = workloads.config2_residual0(n)
    res_ref = res_gpu.copy()
    comp = binding.Compressor(n, [10.0, 100.0, 1000.0], 1)
    for it in range(5):
        g = workloads.config2_grad(it, n)
        gpu = gpu_compress(g, res_gpu, [10.0, 100.0, 1000.0], 1, comp=comp)
        ref = oracle_compress(g, res_ref, [10.0, 100.0, 1000.0], 1)
        assert_same(gpu, ref, f"config2 it{it}")
        assert gpu[4] == {"any_fallback": 0, "fallback_segments": 0, "internal_error": 0, "segments": 1,
                          "narrow_fallback_segments": 0}
        res_gpu, res_ref = gpu[3], ref[3]


def test_config3_reduced_five_iterations():
    n_conv, n_fc = 300_000, 2_500_007
    n = n_conv + n_fc
    res_gpu = np.zeros(n, np.float32)
    res_ref = np.zeros(n, np.float32)
    comp = binding.Compressor(n, [1000.0])
    for it in range(5):
        g = workloads.config3_grad(it, n_conv, n_fc)
        gpu = gpu_compress(g, res_gpu, [1000.0], comp=comp)
        ref = oracle_compress(g, res_ref, [1000.0])
        assert_same(gpu, ref, f"config3 it{it}")
        assert gpu[4]["internal_error"] == 0
        res_gpu, res_ref = gpu[3], ref[3]


def test_config4_reduced():
    g = workloads.config4_grad(0, vocab=3000, hidden=130)   # 95 % of embedding rows exactly zero
    z = np.zeros(g.size, np.float32)
    for commit in (0, 1):
        check(g, z, [100.0, 1000.0], commit=commit, what=f"config4 commit={commit}")


# --------------------------------------------------------------------------
# layerwise (segmented) mode
# --------------------------------------------------------------------------

@pytest.mark.parametrize("flags", [0, FB])
def test_segmented_ragged(flags):
    sizes = [64, 1, 4096, 37, 100_003, 2, 9408, 64, 64, 1000, 4097, 8191, 3, 250_001, 5]
    off = workloads.offsets_of(sizes)
    n = int(off[-1])
    g = workloads.resnet_like_gradient(n, seed=61)
    r = workloads.normal_gradient(n, 1e-5, seed=62)
    check(g, r, [100.0], seg=off, flags=flags, what="segmented cf100")
    check(g, r, [10.0, 100.0, 1000.0], commit=0, seg=off, flags=flags, what="segmented 3 CFs")


def test_layerwise_small_tensors_only_and_at_the_size_limit():
    """Tensors of at most 8192 elements are selected by one workgroup each, out of LDS: a call that has only such
    tensors (no tile at all), tensors just below, at and above the limit, ties, several CFs, every commit."""
    rng = np.random.default_rng(5)
    for sizes in ([64, 1, 100, 8192, 5, 2048, 4097], [8192, 8193, 8191, 16_384, 3, 70_001, 8192]):
        off = workloads.offsets_of(sizes)
        n = int(off[-1])
        g = workloads.resnet_like_gradient(n, seed=n)
        r = workloads.normal_gradient(n, 1e-5, seed=n + 1)
        check(g, r, [100.0], seg=off, what=f"small tensors {sizes}")
        for commit in range(3):
            check(g, r, [1.0, 7.0, 100.0], commit=commit, seg=off, what=f"small tensors {sizes} commit {commit}")
        ties = (rng.integers(-4, 5, n) * 0.5).astype(np.float32)
        ties[rng.random(n) < 0.2] = -0.0
        check(ties, np.zeros(n, np.float32), [3.0, 20.0], commit=0, seg=off, what=f"small tensors, ties {sizes}")
        check(ties, np.zeros(n, np.float32), [3.0, 20.0], commit=1, seg=off, what=f"small tensors, ties {sizes}")


def test_config5_reduced_resnet_tensor_list():
    sizes = workloads.scaled_sizes(workloads.resnet101_tensor_sizes(), 16)
    off = workloads.offsets_of(sizes)
    n = int(off[-1])
    assert len(sizes) == 314
    g = workloads.config5_worker_grad(0, n)
    gpu, ref = check(g, np.zeros(n, np.float32), [100.0], seg=off, what="config5 reduced")
    assert gpu[2].shape == (314, 1, 4)
    assert gpu[0].size == sum(-(-s // 100) for s in sizes)


# --------------------------------------------------------------------------
# determinism, workspace reuse, buffers left alone
# --------------------------------------------------------------------------

def test_repeat_runs_are_bit_identical_and_grad_is_untouched():
    n = 1_500_000
    g = workloads.resnet_like_gradient(n, seed=71)
    r = workloads.normal_gradient(n, 1e-5, seed=72)
    comp = binding.Compressor(n, [10.0, 100.0], 1)
    gt = torch.from_numpy(g).cuda()
    first = None
    for rep in range(5):
        rt = torch.from_numpy(r.copy()).cuda()
        idx, val, stats = comp(gt, rt)
        torch.cuda.synchronize()
        out = (idx.cpu().numpy().copy(), val.cpu().numpy().copy(), stats.cpu().numpy().copy(), rt.cpu().numpy())
        if first is None:
            first = out
        else:
            for a, b in zip(first, out):
                assert np.array_equal(a.view(np.uint8), b.view(np.uint8))
    assert np.array_equal(gt.cpu().numpy(), g)


# --------------------------------------------------------------------------
# decompression
# --------------------------------------------------------------------------

def _decompress_case(n, ks, seed, offset_elems=0, common=0, alpha=None):
    from oracle import oracle
    rng = np.random.default_rng(seed)
    idxs, vals = [], []
    shared = rng.choice(n, size=common, replace=False)     # indices every worker's message holds
    for k in ks:
        own = rng.choice(n, size=k, replace=False)
        own = np.setdiff1d(own, shared)[:max(k - common, 0)]
        idxs.append(np.sort(np.concatenate([shared[:min(common, k)], own])).astype(np.int32))
        vals.append(rng.standard_normal(idxs[-1].size).astype(np.float32))
    ks = [i.size for i in idxs]
    idx = np.concatenate(idxs) if ks else np.zeros(0, np.int32)
    val = np.concatenate(vals) if ks else np.zeros(0, np.float32)
    dense = rng.standard_normal(n).astype(np.float32)
    want = dense.copy()
    if alpha is None:
        oracle.decompress_accumulate(idx, val, ks, want)
    else:
        oracle.decompress_update(idx, val, ks, alpha, want)
    # without a workspace (tile boundaries by search) and with one (boundaries computed once)
    for ws in (None, torch.empty(binding.gravac_decompress_workspace_bytes(len(ks), n), dtype=torch.uint8, device="cuda")):
        if ws is not None:
            ws.fill_(0xA5)                                  # the contents on entry do not matter
        buf = torch.zeros(n + offset_elems, dtype=torch.float32, device="cuda")
        d = buf[offset_elems:]
        d.copy_(torch.from_numpy(dense))
        di, dv = torch.from_numpy(idx).cuda(), torch.from_numpy(val).cuda()
        if alpha is None:
            binding.gravac_decompress_accumulate(di, dv, ks, d, workspace=ws)
        else:
            binding.gravac_decompress_update(di, dv, ks, alpha, d, workspace=ws)
        torch.cuda.synchronize()
        got = d.cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), "workspace" if ws is not None else "search"
        if offset_elems:
            assert float(buf[:offset_elems].abs().sum()) == 0.0


def test_decompress_accumulate_small_and_ragged():
    _decompress_case(1000, [100, 0, 250, 1000, 7], seed=1)
    _decompress_case(8192, [8192], seed=2)
    _decompress_case(8193, [1, 8193], seed=3)
    _decompress_case(100_003, [5000] * 8, seed=4)
    _decompress_case(100_003, [5000] * 8, seed=5, offset_elems=1)     # dense buffer not 16-byte aligned
    _decompress_case(50_000, [100] * 70, seed=6)                       # more than 64 workers: two launches


def test_decompress_tiles_with_few_pairs():
    # tiles of 8192 entries with a handful of pairs each take another route through the kernel (only the named
    # entries are read and written) than tiles with many; the same entry named by several workers must still be
    # added to in worker order
    _decompress_case(1_000_003, [300] * 8, seed=11, common=120)
    _decompress_case(1_000_003, [300] * 8, seed=12, common=120, offset_elems=3)
    _decompress_case(200_000, [40] * 64, seed=13, common=25)           # 64 workers, about 100 pairs per tile
    _decompress_case(300_000, [30] * 70, seed=14, common=10)           # two launches
    _decompress_case(81_920, [640] * 8, seed=15, common=300)           # about 512 pairs per tile: both routes in one call
    _decompress_case(81_920 + 77, [64, 0, 1, 640, 0, 3, 512, 9], seed=16, common=0)
    _decompress_case(5, [5, 5, 5], seed=17, common=5)


def test_decompress_update_is_the_sgd_step_from_the_messages():
    # Alg. 1's update w - eta * aggregate applied pair by pair (alpha = -eta / W): dense and sparse tiles, entries named
    # by several workers, ragged sizes, an unaligned buffer, more than 64 workers, and multipliers whose products round
    for alpha in (-0.1 / 8, 1.0 + 2.0 ** -12, -3.0):
        _decompress_case(100_003, [5000] * 8, seed=21, common=2000, alpha=alpha)
        _decompress_case(1_000_003, [300] * 8, seed=22, common=120, alpha=alpha)
    _decompress_case(81_920 + 77, [64, 0, 1, 640, 0, 3, 512, 9], seed=23, alpha=-0.0125, offset_elems=1)
    _decompress_case(300_000, [30] * 70, seed=24, common=10, alpha=0.5)
    _decompress_case(8192, [8192, 8192], seed=25, common=8192, alpha=-1e-3)
    _decompress_case(1000, [100, 0, 250, 1000, 7], seed=26, alpha=0.0)       # x + (+-0) = x


def test_decompress_gaps_clusters_and_out_of_range_indices():
    from oracle import oracle
    n = 600_000
    rng = np.random.default_rng(77)
    # worker 0: one cluster at the start; worker 1: one pair at the very end; worker 2: empty; worker 3: two clusters
    # far apart; worker 4: every 8192-th element (one pair per tile)
    parts = [np.arange(0, 5000), np.array([n - 1]), np.zeros(0, np.int64),
             np.concatenate([np.arange(100_000, 103_000), np.arange(590_000, 591_000)]), np.arange(0, n, 8192)]
    idx = np.concatenate(parts).astype(np.int32)
    val = rng.standard_normal(idx.size).astype(np.float32)
    ks = [p.size for p in parts]
    dense = rng.standard_normal(n).astype(np.float32)
    want = dense.copy()
    oracle.decompress_accumulate(idx, val, ks, want)
    for ws in (None, torch.empty(binding.gravac_decompress_workspace_bytes(len(ks), n), dtype=torch.uint8, device="cuda")):
        d = torch.from_numpy(dense).cuda()
        binding.gravac_decompress_accumulate(torch.from_numpy(idx).cuda(), torch.from_numpy(val).cuda(), ks, d, workspace=ws)
        assert np.array_equal(d.cpu().numpy().view(np.uint32), want.view(np.uint32))
    # indices outside [0, n) are ignored (the oracle rejects them, so the expectation is built by hand)
    idx2 = np.array([-5, -1, 0, 7, n - 1, n, n + 100], np.int32)
    val2 = np.arange(1, 8, dtype=np.float32)
    want2 = dense.copy()
    for i, v in zip(idx2, val2):
        if 0 <= i < n:
            want2[i] += v
    for ws in (None, torch.empty(binding.gravac_decompress_workspace_bytes(1, n), dtype=torch.uint8, device="cuda")):
        d = torch.from_numpy(dense).cuda()
        binding.gravac_decompress_accumulate(torch.from_numpy(idx2).cuda(), torch.from_numpy(val2).cuda(), [7], d, workspace=ws)
        assert np.array_equal(d.cpu().numpy().view(np.uint32), want2.view(np.uint32))
    with pytest.raises(binding.GravacError) as e:
        binding.gravac_decompress_accumulate(torch.from_numpy(idx2).cuda(), torch.from_numpy(val2).cuda(), [7], d,
                                             workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.code == binding.ERR_WORKSPACE


def test_decompress_sparse_and_dense_regimes():
    _decompress_case(3_000_000, [3000] * 8, seed=7)                    # most tiles untouched
    _decompress_case(1_000_000, [100_000] * 8, seed=8)                 # every tile touched by every worker


def test_compress_then_decompress_eight_workers():
    """Reduced twin of configuration 5: eight workers' layerwise messages summed into one dense buffer."""
    from oracle import oracle
    sizes = workloads.scaled_sizes(workloads.resnet101_tensor_sizes(), 32)
    off = workloads.offsets_of(sizes)
    n = int(off[-1])
    comp = binding.Compressor(n, [100.0], 0, off)
    k = comp.k_total
    all_idx = torch.empty(8 * k, dtype=torch.int32, device="cuda")
    all_val = torch.empty(8 * k, dtype=torch.float32, device="cuda")
    ref_idx, ref_val = [], []
    for w in range(8):
        g = workloads.config5_worker_grad(w, n)
        z = np.zeros(n, np.float32)
        gpu = gpu_compress(g, z, [100.0], 0, off, comp=comp)
        ref = oracle_compress(g, z, [100.0], 0, off)
        assert_same(gpu, ref, f"worker {w}")
        all_idx[w * k:(w + 1) * k] = comp.out_idx
        all_val[w * k:(w + 1) * k] = comp.out_val
        ref_idx.append(ref[0]), ref_val.append(ref[1])
    dense = torch.zeros(n, dtype=torch.float32, device="cuda")
    binding.gravac_decompress_accumulate(all_idx, all_val, [k] * 8, dense,
                                         workspace=torch.empty(binding.gravac_decompress_workspace_bytes(8, n), dtype=torch.uint8,
                                                               device="cuda"))
    torch.cuda.synchronize()
    want = np.zeros(n, np.float32)
    oracle.decompress_accumulate(np.concatenate(ref_idx), np.concatenate(ref_val), [k] * 8, want)
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), want.view(np.uint32))


# --------------------------------------------------------------------------
# iterative use: many calls on one workspace, whose contents are whatever the previous call left
# --------------------------------------------------------------------------

def _iterate(n, cfs, commit, grads, flags_per_it, seg=None, comp=None, res0=None, carry=True):
    """Run consecutive calls carrying the residual; compare every call with the oracle; return the statuses."""
    comp = comp or binding.Compressor(n, cfs, commit, seg)
    res_gpu = np.zeros(n, np.float32) if res0 is None else res0.copy()
    res_ref = res_gpu.copy()
    out = []
    for it, (g, fl) in enumerate(zip(grads, flags_per_it)):
        gpu = gpu_compress(g, res_gpu, cfs, commit, seg, flags=fl, comp=comp)
        ref = oracle_compress(g, res_ref, cfs, commit, seg)
        assert_same(gpu, ref, f"iteration {it}")
        assert gpu[4]["internal_error"] == 0
        out.append(gpu[4])
        if carry:
            res_gpu, res_ref = gpu[3], ref[3]
    return out, comp


def test_iterations_on_one_workspace():
    n = 1_200_003
    grads = [workloads.config3_grad(it, 150_000, n - 150_000) for it in range(5)]
    st, _ = _iterate(n, [1000.0], 0, grads, [0] * 5)
    assert [s["any_fallback"] for s in st] == [0] * 5
    # three CFs on the Laplace-with-outliers gradient, residual carried: the thresholds keep moving (one of them sits
    # among a thousand outliers); whichever route each call takes, the results are the oracle's
    grads = [workloads.config2_grad(it, n) for it in range(5)]
    _iterate(n, [10.0, 100.0, 1000.0], 1, grads, [0, 0, FB, 0, 0], res0=workloads.config2_residual0(n))


def test_one_workspace_other_cf_list_and_lost_contents():
    n = 500_001
    g = [workloads.normal_gradient(n, 1e-3, seed=s) for s in range(4)]
    st, comp = _iterate(n, [100.0], 0, g[:1], [0])
    assert st[0]["any_fallback"] == 0
    # the same workspace with another CF list, then with its contents overwritten: every call starts from scratch
    comp2 = binding.Compressor(n, [50.0], 0)
    comp2.workspace = comp.workspace
    st, _ = _iterate(n, [50.0], 0, g[1:3], [0, 0], comp=comp2, carry=False)
    assert [s["any_fallback"] for s in st] == [0, 0]
    comp2.workspace.fill_(0xA5)
    st, _ = _iterate(n, [50.0], 0, g[3:], [0], comp=comp2, carry=False)
    assert st[0]["any_fallback"] == 0


def test_flat_call_with_the_larger_sample_in_blocks_of_two_groups():
    """k n large enough (k = n = 12 M for the CF 1 of the list) for the flat sampling pass to take more than 131,072
    samples, in blocks of 2048: the form of the sampling kernel between the plain one and the one the full-size
    VGG16-shaped test at CF 10 runs."""
    n = 12_000_000
    g = workloads.normal_gradient(n, 1e-3, seed=410)
    r = workloads.normal_gradient(n, 3e-4, seed=411)
    check(g, r, [1.0, 3.0], 1, what="cf 3 committed", expect_fallback=False)
    check(g, r, [1.0, 3.0], 0, what="cf 1 committed")


def test_a_cf_that_selects_millions_next_to_a_sparse_one():
    """CF 4 on 12 M elements (k = 3 M: the sub-tiles are mostly candidates and keep no candidate list) in one call
    with CF 1000, either of them committed, the residual carried."""
    n = 12_000_000
    grads = [workloads.normal_gradient(n, 1e-3, seed=400 + it) for it in range(3)]
    _iterate(n, [4.0, 1000.0], 0, grads, [0, 0, 0])
    _iterate(n, [4.0, 1000.0], 1, grads, [0, 0, 0])
    st, _ = _iterate(n, [4.0, 1000.0], 0, grads, [0, 0, 0], carry=False)
    assert [s["any_fallback"] for s in st] == [0, 0, 0]


def test_scale_jumps_between_iterations():
    n = 800_000
    grads = [workloads.normal_gradient(n, 1e-3, seed=1), workloads.normal_gradient(n, 1e-3, seed=2),
             workloads.normal_gradient(n, 2e-2, seed=3),      # twenty times larger
             workloads.normal_gradient(n, 2e-2, seed=4),
             workloads.normal_gradient(n, 1e-4, seed=5)]      # far smaller
    st, _ = _iterate(n, [100.0], 0, grads, [0] * 5, carry=False)
    assert [s["any_fallback"] for s in st] == [0] * 5
    _iterate(n, [100.0], 0, grads, [0] * 5)


def test_iterations_layerwise():
    sizes = [64, 4096, 37, 100_003, 9408, 64, 1000, 40_970, 250_001, 5]
    off = workloads.offsets_of(sizes)
    n = int(off[-1])
    grads = [workloads.normal_gradient(n, 1e-3, seed=80 + it) for it in range(3)]
    st, _ = _iterate(n, [10.0], 0, grads, [0, 0, 0], seg=off, carry=False)
    assert st[1]["any_fallback"] == 0 and st[2]["any_fallback"] == 0
    # a distribution whose threshold sits in a gap (1 % outliers at CF 100) and a carried residual
    grads = [workloads.resnet_like_gradient(n, seed=90 + it) for it in range(3)]
    _iterate(n, [100.0], 0, grads, [0, FB, 0], seg=off)


def test_dense_and_sparse_sub_tiles_in_one_call():
    """VGG16-like mix at CF 10: the conv part's sub-tiles are mostly candidates (read again by the emit step, no
    candidate list), the fc part's hold a few; the boundary between the parts falls inside a sub-tile."""
    n_conv, n_fc = 301_111, 2_000_003
    n = n_conv + n_fc
    grads = [workloads.config3_grad(it, n_conv, n_fc) for it in range(3)]
    for cfs, commit in (([10.0], 0), ([10.0, 1000.0], 0), ([10.0, 1000.0], 1), ([2.0], 0)):
        _iterate(n, cfs, commit, grads, [0, 0, FB])


@pytest.mark.parametrize("off_g,off_r", [(1, 1), (2, 3), (3, 0), (0, 2)])
def test_buffers_at_any_float_boundary(off_g, off_r):
    """grad and residual that do not start at a multiple of 16 bytes (slices of a larger buffer): same results."""
    n = 300_007
    g = workloads.resnet_like_gradient(n, seed=5)
    r = workloads.normal_gradient(n, 1e-5, seed=6)
    bg = torch.zeros(n + 8, dtype=torch.float32, device="cuda")
    br = torch.zeros(n + 8, dtype=torch.float32, device="cuda")
    for cfs, commit, seg in (([100.0], 0, None), ([2.0, 50.0], 0, None), ([10.0], 0, workloads.offsets_of([1001, 200_000, 99_006]))):
        gt, rt = bg[off_g:off_g + n], br[off_r:off_r + n]
        gt.copy_(torch.from_numpy(g))
        rt.copy_(torch.from_numpy(r))
        comp = binding.Compressor(n, cfs, commit, seg)
        idx, val, stats = comp(gt, rt)
        torch.cuda.synchronize()
        assert comp.status()["internal_error"] == 0
        ref = oracle_compress(g, r, cfs, commit, seg)
        gpu = (idx.cpu().numpy(), val.cpu().numpy(), stats.cpu().numpy(), rt.cpu().numpy())
        assert_same(gpu, ref, f"offsets {off_g}, {off_r}, cfs {cfs}")
        # nothing outside the slices was written
        assert float(bg[:off_g].abs().sum()) == 0.0 and float(bg[off_g + n:].abs().sum()) == 0.0
        assert float(br[:off_r].abs().sum()) == 0.0 and float(br[off_r + n:].abs().sum()) == 0.0


def test_mass_of_equal_values_at_the_threshold_over_several_scan_slices():
    """More ties at the threshold than a gather list holds, in a gradient long enough for several slices of the
    scan (4096 tiles each): the located bin is histogrammed key by key and the tiles' ties are counted again."""
    n = 40_000_000
    rng = np.random.default_rng(123)
    g = (rng.integers(-3, 4, n) * 0.25).astype(np.float32)
    r = np.zeros(n, np.float32)
    for cf in (3.0, 20.0):
        check(g, r, [cf], what=f"ties over slices cf={cf}")


def test_values_on_a_coarse_grid_and_the_repairs_of_the_zeroed_entries():
    """Gradients whose values sit on a grid of 8 mantissa bits (what a bfloat16 backward pass hands over): a sample
    bin then holds one or two distinct keys, so the key from which the pass zeroes listed entries lands on either
    side of the threshold, with ties at it.  Both repairs of the emit step (a selected entry below that key gets
    +0, an unselected one at or above it gets acc back) are exercised over iterations, flat and layerwise."""
    n = 2_500_003
    rng = np.random.default_rng(77)

    def on_grid(x):
        b = x.astype(np.float32).view(np.uint32)
        return ((b + 0x8000) & 0xFFFF0000).astype(np.uint32).view(np.float32)

    grads = [on_grid(rng.laplace(0.0, 1e-4, n)) for _ in range(3)]
    for cfs, commit in (([10.0], 0), ([100.0], 0), ([7.0, 300.0], 0), ([7.0, 300.0], 1)):
        _iterate(n, cfs, commit, grads, [0, 0, 0])
    seg = workloads.offsets_of([100_000, 9_000, 1_200_003, 191_000, 1_000_000])
    res_gpu = np.zeros(n, np.float32)
    res_ref = np.zeros(n, np.float32)
    for it in range(3):
        gpu = gpu_compress(grads[it], res_gpu, [20.0], seg=seg)
        ref = oracle_compress(grads[it], res_ref, [20.0], seg=seg)
        assert_same(gpu, ref, f"grid values, layerwise, it{it}")
        res_gpu, res_ref = gpu[3], ref[3]
