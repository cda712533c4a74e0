"""GPU parity of compression without commit (GRAVAC_FLAG_NO_COMMIT) and of the protocol built on it: Alg. 1 evaluates
theta_min and a candidate CF and sends one of the two messages, so nothing is removed from the residual until the
decision is known (compress without commit, second-level Top-k on the message, gravac_commit of the message sent).

Expected values come from the oracle alone: the message and the statistics are those of the ordinary call, and acc is
the oracle's residual with the oracle's message put back (message + residual = acc bitwise, a pinned invariant).
"""
import numpy as np
import pytest
import torch

from paper_2305_12201_amd import binding, workloads
from tests.gpu_util import assert_same, gpu_compress, oracle_compress

pytestmark = pytest.mark.gpu

NC = binding.FLAG_NO_COMMIT
FB = binding.FLAG_FORCE_FALLBACK


def acc_of(ref):
    idx, val, _, res = ref
    acc = res.copy()
    acc[idx] = val
    return acc


def check_no_commit(g, r, cfs, commit=0, seg=None, flags=0, what=""):
    gpu = gpu_compress(g, r, cfs, commit, seg, flags=flags | NC)
    ref = oracle_compress(g, r, cfs, commit, seg)
    assert gpu[4]["internal_error"] == 0, what
    assert_same(gpu, (ref[0], ref[1], ref[2], acc_of(ref)), what)


@pytest.mark.parametrize("n", [1, 70, 8192, 8193, 100_003, 1_300_001])
def test_flat_every_regime(n):
    g = workloads.normal_gradient(n, 1e-3, seed=n)
    r = workloads.normal_gradient(n, 1e-4, seed=n + 1)
    for cf in (1.0, 2.0, 10.0, 300.0):   # CF 1 and 2: sub-tiles without a candidate list
        check_no_commit(g, r, [cf], what=f"n={n} cf={cf}")
    check_no_commit(g, r, [5.0], flags=FB, what=f"n={n} exact route")


def test_several_cfs_ties_and_layerwise_with_small_tensors():
    n = 700_001
    rng = np.random.default_rng(3)
    g = (rng.integers(-4, 5, n) * 0.125).astype(np.float32)     # heavy ties, signed zeros among the selected
    g[rng.integers(0, n, 1000)] = -0.0
    r = np.zeros(n, np.float32)
    for commit in (0, 1, 2):
        check_no_commit(g, r, [3.0, 40.0, 900.0], commit, what=f"ties commit {commit}")
    g = workloads.resnet_like_gradient(n, seed=9)
    r = workloads.normal_gradient(n, 1e-5, seed=10)
    seg = workloads.offsets_of([5, 8192, 300_000, 64, 391_740])
    check_no_commit(g, r, [20.0], seg=seg, what="layerwise")
    check_no_commit(g, r, [20.0, 200.0], 1, seg=seg, what="layerwise, two CFs")


def test_random_k_without_commit():
    n = 500_009
    g = workloads.normal_gradient(n, 1e-3, seed=21)
    r = workloads.normal_gradient(n, 1e-4, seed=22)
    from oracle import oracle
    comp = binding.Compressor(n, [50.0], 0)
    dg, dr = torch.from_numpy(g).cuda(), torch.from_numpy(r.copy()).cuda()
    idx, val, stats = comp.randomk(dg, dr, seed=77, flags=NC)
    torch.cuda.synchronize()
    res = r.copy()
    oi, ov, os_ = oracle.randomk_compress(g, res, [50.0], 77)
    acc = res.copy(); acc[oi] = ov
    assert np.array_equal(idx.cpu().numpy(), oi) and np.array_equal(val.cpu().numpy().view(np.uint32), ov.view(np.uint32))
    assert np.array_equal(dr.cpu().numpy().view(np.uint32), acc.view(np.uint32))


def test_decide_after_both_messages_are_known():
    """compress at theta_min without commit -> candidate message from that message -> commit of the one that is sent:
    the residual equals that of a direct compression at the CF sent (Sec. IV-C), whichever is sent."""
    n = 1_500_007
    g = workloads.resnet_like_gradient(n, seed=31)
    r0 = workloads.normal_gradient(n, 1e-5, seed=32)
    theta_min, rel = 10.0, 16.0
    for send_candidate in (True, False):
        dg, dr = torch.from_numpy(g).cuda(), torch.from_numpy(r0.copy()).cuda()
        comp = binding.Compressor(n, [theta_min], 0)
        i1, v1, _ = comp(dg, dr, flags=NC)
        k2 = binding.gravac_topk_count(i1.numel(), rel)
        ws = torch.empty(binding.gravac_workspace_bytes(i1.numel(), 1, 0), dtype=torch.uint8, device="cuda")
        i2 = torch.empty(k2, dtype=torch.int32, device="cuda")
        v2 = torch.empty(k2, dtype=torch.float32, device="cuda")
        st2 = torch.zeros(1, 4, dtype=torch.float64, device="cuda")
        binding.gravac_recompress(i1, v1, rel, None, None, out_idx=i2, out_val=v2, out_stats=st2, workspace=ws)
        binding.gravac_commit(i2 if send_candidate else i1, dr)
        torch.cuda.synchronize()
        cf_sent = theta_min * rel if send_candidate else theta_min
        ref = oracle_compress(g, r0, [cf_sent])
        sent_i, sent_v = (i2, v2) if send_candidate else (i1, v1)
        assert np.array_equal(sent_i.cpu().numpy(), ref[0]), cf_sent
        assert np.array_equal(sent_v.cpu().numpy().view(np.uint32), ref[1].view(np.uint32)), cf_sent
        assert np.array_equal(dr.cpu().numpy().view(np.uint32), ref[3].view(np.uint32)), cf_sent


def test_flag_is_refused_where_it_has_no_meaning():
    n = 10_000
    g = torch.from_numpy(workloads.normal_gradient(n, 1e-3, seed=1)).cuda()
    r = torch.zeros(n, dtype=torch.float32, device="cuda")
    comp = binding.Compressor(n, [10.0], 0)
    i1, v1, _ = comp(g, r)
    ws = torch.empty(binding.gravac_workspace_bytes(i1.numel(), 1, 0), dtype=torch.uint8, device="cuda")
    oi = torch.empty(i1.numel(), dtype=torch.int32, device="cuda")
    ov = torch.empty(i1.numel(), dtype=torch.float32, device="cuda")
    st = torch.zeros(1, 4, dtype=torch.float64, device="cuda")
    with pytest.raises(binding.GravacError):
        binding.gravac_recompress(i1, v1, 2.0, None, r, out_idx=oi, out_val=ov, out_stats=st, workspace=ws, flags=NC)
    with pytest.raises(binding.GravacError):
        comp(g, r, flags=4)
