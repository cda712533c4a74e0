"""Pins for the oracle's threshold sparsifier (Sec. II-C: the selection rule the paper gives for DGC, entries
below a threshold are discarded; with error feedback, Sec. III-B).  Every check is independent of the oracle's code:
a Python loop on tiny inputs, numpy's float32 add and comparisons, the oracle's Top-k (itself pinned elsewhere) at
the threshold equal to its k-th magnitude, invariants, monotonicity."""
import numpy as np
import pytest

from oracle import oracle
from paper_2305_12201_amd import workloads


def _mag(a):
    return a.view(np.uint32) & np.uint32(0x7FFFFFFF)


def _loop_reference(grad, residual, tau):
    """Element by element, in plain Python."""
    idx, val, res = [], [], []
    ss_sel = ss_all = 0.0
    for i in range(grad.size):
        a = np.float32(residual[i]) + np.float32(grad[i])
        ss_all += float(a) * float(a)
        if abs(float(a)) >= float(np.float32(tau)):       # no NaN in these inputs
            idx.append(i); val.append(a); res.append(np.float32(0.0)); ss_sel += float(a) * float(a)
        else:
            res.append(a)
    return np.array(idx, np.int32), np.array(val, np.float32), np.array(res, np.float32), ss_sel, ss_all


@pytest.mark.parametrize("seed", range(6))
def test_against_a_python_loop_with_ties_signed_zeros_and_entries_equal_to_tau(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 400))
    g = (rng.integers(-8, 9, n) * 0.25).astype(np.float32)
    r = (rng.integers(-2, 3, n) * 0.25).astype(np.float32)
    g[rng.random(n) < 0.1] = -0.0
    for tau in (0.25, 0.5, 1.0, 1.25, 2.75, 100.0):
        res = r.copy()
        idx, val, stats, count = oracle.threshold_compress(g, res, tau)
        wi, wv, wr, ss_sel, ss_all = _loop_reference(g, r, tau)
        assert count == wi.size and np.array_equal(idx, wi)
        assert np.array_equal(val.view(np.uint32), wv.view(np.uint32))
        assert np.array_equal(res.view(np.uint32), wr.view(np.uint32))          # kept slots are +0, not -0
        np.testing.assert_allclose(stats[:2], [ss_sel, ss_all], rtol=1e-12)
        assert stats[2] == (1.0 if ss_all == 0.0 else ss_sel / ss_all) or abs(stats[2] - ss_sel / ss_all) < 1e-12
        assert stats[3] == float(np.float32(tau))


def test_numpy_definition_and_invariants_on_a_gradient_like_input():
    n = 200_003
    g = workloads.resnet_like_gradient(n, seed=3)
    r = workloads.normal_gradient(n, 1e-5, seed=4)
    acc = r + g                                             # numpy's binary32 add
    prev = None
    for tau in (1e-6, 1e-4, 3e-4, 1e-2, 1.0):
        res = r.copy()
        idx, val, stats, count = oracle.threshold_compress(g, res, tau)
        keep = np.abs(acc) >= np.float32(tau)
        assert np.array_equal(idx, np.nonzero(keep)[0].astype(np.int32))
        assert np.array_equal(val.view(np.uint32), acc[keep].view(np.uint32))
        # message + residual = acc, bit for bit; nothing below tau in the message, nothing at or above it left
        back = res.copy(); back[idx] = val
        assert np.array_equal(back.view(np.uint32), acc.view(np.uint32))
        assert np.all(res[idx].view(np.uint32) == 0)
        assert count == 0 or np.abs(val).min() >= np.float32(tau)
        assert np.abs(res).max() < np.float32(tau)
        ss_all = float(np.dot(acc.astype(np.float64), acc.astype(np.float64)))
        ss_sel = float(np.dot(val.astype(np.float64), val.astype(np.float64)))
        np.testing.assert_allclose(stats[:3], [ss_sel, ss_all, ss_sel / ss_all], rtol=1e-10)
        assert 0.0 <= stats[2] <= 1.0
        if prev is not None:                                # a higher threshold keeps a subset and loses gain
            assert set(idx.tolist()) <= prev[0] and stats[2] <= prev[1]
        prev = (set(idx.tolist()), stats[2])
    assert prev[0] == set() and prev[1] == 0.0              # tau above every magnitude: empty message, gain 0


def test_equals_topk_at_the_threshold_of_its_kth_magnitude():
    """Top-k at k keeps the k largest; the threshold rule at tau = the k-th largest magnitude keeps those and every
    further entry equal to tau.  Without ties at tau the two messages, residuals and gains are the same."""
    n = 50_000
    g = workloads.normal_gradient(n, 1e-3, seed=11)         # continuous values: no ties
    r = workloads.normal_gradient(n, 1e-4, seed=12)
    for cf in (10.0, 100.0, 1000.0):
        res_k = r.copy()
        ik, vk, sk = oracle.compress(g, res_k, [cf])
        tau = float(sk[0, 0, 3])                            # |acc| of the smallest selected entry
        res_t = r.copy()
        it, vt, st, count = oracle.threshold_compress(g, res_t, tau)
        assert count == ik.size and np.array_equal(it, ik)
        assert np.array_equal(vt.view(np.uint32), vk.view(np.uint32))
        assert np.array_equal(res_t.view(np.uint32), res_k.view(np.uint32))
        np.testing.assert_allclose(st[:3], sk[0, 0, :3], rtol=1e-12)
    # with ties at tau the threshold rule keeps them all, Top-k only the lowest indices
    g = (np.arange(40) % 4).astype(np.float32)              # magnitudes 0, 1, 2, 3, ten of each
    z = np.zeros(40, np.float32)
    ik, _, sk = oracle.compress(g, z.copy(), [40.0 / 15.0])  # k = 15: the ten 3s and five of the 2s
    assert ik.size == 15 and sk[0, 0, 3] == 2.0
    it, _, _, count = oracle.threshold_compress(g, z.copy(), 2.0)
    assert count == 20 and set(ik.tolist()) < set(it.tolist())


def test_capacity_denormals_and_bad_arguments():
    n = 1000
    g = workloads.normal_gradient(n, 1.0, seed=5)
    r = np.zeros(n, np.float32)
    full = oracle.threshold_compress(g, r.copy(), 0.5)
    res = r.copy()
    idx, val, stats, count = oracle.threshold_compress(g, res, 0.5, capacity=full[3] - 1)
    assert idx.size == 0 and count == full[3]
    assert np.array_equal(res.view(np.uint32), g.view(np.uint32))            # nothing removed: the residual is acc
    np.testing.assert_allclose(stats, full[2], rtol=0)
    res = r.copy()
    idx, _, _, count = oracle.threshold_compress(g, res, 0.5, capacity=full[3])  # exactly enough
    assert count == full[3] and idx.size == count
    # a denormal threshold and denormal values
    d = np.array([1e-40, -3e-40, 0.0, -0.0, 2e-40, 1e-39], np.float32)
    idx, val, _, count = oracle.threshold_compress(d, np.zeros(6, np.float32), 2e-40)
    assert idx.tolist() == [1, 4, 5] and count == 3
    for bad in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(RuntimeError):
            oracle.threshold_compress(g, r.copy(), bad)
