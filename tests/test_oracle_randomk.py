"""Pins of the Random-k oracle (Sec. II-C names the method; the draw is this build's reading, stated in the
oracle's header): the priority function is a bijection (checked through an inverse written here), the kept
set is what a brute-force rank count over the priorities gives, the draw is uniform and unbiased (selection
frequencies, mean gain = k/n), and the error-feedback bookkeeping is the same as for Top-k."""
import math

import numpy as np

from oracle import oracle
from paper_2305_12201_amd import workloads

M = 0x7FFFFFFF


def _unxorshift(x, s):
    y = x
    for _ in range(31 // s + 1):
        y = x ^ (y >> s)
    return y


def _inverse_priority(seed, r):
    """Inverse of the oracle's priority function, step by step from the end (each step is a bijection)."""
    z = oracle.splitmix64_first(seed)
    s0, s1 = z & M, (z >> 32) & M
    inv = lambda m: pow(m, -1, 1 << 31)
    x = _unxorshift(r, 15)
    x = (x * inv(0x297A2D39)) & M
    x = _unxorshift(x, 15)
    x = (x * inv(0x2C1B3C6D)) & M
    x = _unxorshift(x, 14)
    x = (x - s1) & M
    x = _unxorshift(x, 16)
    x = (x * inv(0x046CA68B)) & M
    x = _unxorshift(x, 15)
    x = (x * inv(0x7FEB352D)) & M
    x = _unxorshift(x, 16)
    return (x - s0) & M


def test_seed_mixing_is_splitmix64():
    # the published generator's first outputs for the seed 1234567 (its reference test vector): stepping the
    # state by the generator's increment gives the following outputs
    gamma = 0x9E3779B97F4A7C15
    want = [6457827717110365317, 3203168211198807973, 9817491932198370423, 4593380528125082431,
            16408922859458223821]
    got = [oracle.splitmix64_first((1234567 + j * gamma) & 0xFFFFFFFFFFFFFFFF) for j in range(5)]
    assert got == want


def test_priority_is_a_bijection_of_31_bit_integers():
    rng = np.random.default_rng(0)
    for seed in (0, 1, 5, 2 ** 40 + 12345, 2 ** 62 - 1):
        idx = [0, 1, 2, M, M - 1] + [int(v) for v in rng.integers(0, M + 1, size=300)]
        for i in idx:
            r = oracle.randomk_priority(seed, i)
            assert 0 <= r <= M
            assert _inverse_priority(seed, r) == i
    # no collision among the first 200,000 indices (a collision would contradict the inverse above)
    pr = np.array([oracle.randomk_priority(77, i) for i in range(200_000)], dtype=np.int64)
    assert np.unique(pr).size == pr.size


def test_priorities_look_uniform():
    pr = np.array([oracle.randomk_priority(3, i) for i in range(100_000)], dtype=np.float64) / 2.0 ** 31
    assert abs(pr.mean() - 0.5) < 0.005 and abs(pr.var() - 1.0 / 12.0) < 0.002
    hist, _ = np.histogram(pr, bins=64, range=(0, 1))
    chi2 = float(((hist - 100_000 / 64) ** 2 / (100_000 / 64)).sum())
    assert chi2 < 64 + 6 * math.sqrt(2 * 64)
    # consecutive indices are not correlated, and another seed gives unrelated priorities
    assert abs(np.corrcoef(pr[:-1], pr[1:])[0, 1]) < 0.01
    pr2 = np.array([oracle.randomk_priority(4, i) for i in range(100_000)], dtype=np.float64) / 2.0 ** 31
    assert abs(np.corrcoef(pr, pr2)[0, 1]) < 0.01


def _brute_force(seed, base, n, k):
    pr = [oracle.randomk_priority(seed, base + i) for i in range(n)]
    return [i for i in range(n) if sum(1 for j in range(n) if pr[j] > pr[i]) < k]


def test_selection_is_the_k_highest_priorities_and_bookkeeping_is_exact():
    n = 1500
    g = workloads.normal_gradient(n, 1e-3, seed=1)
    r0 = workloads.normal_gradient(n, 1e-4, seed=2)
    for cf, seed in ((10.0, 9), (3.0, 10), (1.0, 11), (1000.0, 12), (7.5, 2 ** 50 + 3)):
        res = r0.copy()
        idx, val, st = oracle.randomk_compress(g, res, [cf], seed)
        k = math.ceil(n / cf)
        assert idx.size == k and np.all(np.diff(idx) > 0)
        assert list(idx) == _brute_force(seed, 0, n, k)
        acc = r0 + g
        assert np.array_equal(val.view(np.uint32), acc[idx].view(np.uint32))
        rebuilt = res.copy()
        assert np.all(rebuilt[idx] == 0) and not np.signbit(rebuilt[idx]).any()
        rebuilt[idx] = val
        assert np.array_equal(rebuilt.view(np.uint32), acc.view(np.uint32))
        assert math.isclose(st[0, 0, 0], float((val.astype(np.float64) ** 2).sum()), rel_tol=1e-12)
        assert math.isclose(st[0, 0, 1], float((acc.astype(np.float64) ** 2).sum()), rel_tol=1e-12)
        assert math.isclose(st[0, 0, 2], st[0, 0, 0] / st[0, 0, 1], rel_tol=1e-15)
        assert st[0, 0, 3] == min(oracle.randomk_priority(seed, int(i)) for i in idx)


def test_nested_cfs_and_commit_and_segments():
    n = 20_000
    g = workloads.resnet_like_gradient(n, seed=3)
    z = np.zeros(n, np.float32)
    sels = []
    for commit in range(3):
        res = z.copy()
        idx, val, st = oracle.randomk_compress(g, res, [10.0, 100.0, 1000.0], 42, commit=commit)
        sels.append(set(idx.tolist()))
        single = oracle.randomk_compress(g, z.copy(), [[10.0, 100.0, 1000.0][commit]], 42)
        assert np.array_equal(idx, single[0]) and np.array_equal(st[0, commit], single[2][0, 0])
    assert sels[2] < sels[1] < sels[0]
    # layerwise: every tensor on its own, priorities by the index in the flat gradient
    sizes = [64, 1, 4096, 37, 10_003, 5799]
    off = workloads.offsets_of(sizes)
    res = z.copy()
    idx, val, st = oracle.randomk_compress(g, res, [10.0], 42, seg_offsets=off)
    at = 0
    for t, s in enumerate(sizes):
        k = math.ceil(s / 10)
        part = idx[at:at + k]
        assert np.all((part >= off[t]) & (part < off[t + 1]))
        pr = np.array([oracle.randomk_priority(42, int(off[t]) + i) for i in range(s)])
        want = np.sort(np.argsort(-pr, kind="stable")[:k]) + off[t]
        assert np.array_equal(part, want)
        at += k
    assert at == idx.size and st.shape == (len(sizes), 1, 4)


def test_draw_is_uniform_and_the_gain_is_unbiased():
    n, cf, seeds = 2000, 10.0, 1500
    k = math.ceil(n / cf)
    g = workloads.normal_gradient(n, 1.0, seed=5)
    z = np.zeros(n, np.float32)
    freq = np.zeros(n)
    pair = 0
    gains = []
    for s in range(seeds):
        idx, _, st = oracle.randomk_compress(g, z.copy(), [cf], 1000 + s)
        freq[idx] += 1
        pair += int(np.isin(idx + 1, idx).sum())
        gains.append(st[0, 0, 2])
    p = k / n
    # every index is kept with probability k/n
    zscore = (freq - seeds * p) / math.sqrt(seeds * p * (1 - p))
    assert abs(zscore.mean()) < 0.1 and 0.85 < zscore.std() < 1.15 and np.abs(zscore).max() < 5.5
    # neighbours are kept together about p^2 of the time
    expect = seeds * (n - 1) * p * (k - 1) / (n - 1)
    assert abs(pair - expect) < 5 * math.sqrt(expect)
    # E[gain] = k/n for a uniformly drawn subset
    assert abs(np.mean(gains) - p) < 4 * np.std(gains) / math.sqrt(seeds)
    # all magnitudes equal: the gain is k/n exactly, whatever is drawn
    ones = np.ones(n, np.float32)
    _, _, st = oracle.randomk_compress(ones, z.copy(), [cf], 7)
    assert st[0, 0, 2] == k / n


def test_error_feedback_sends_everything_eventually():
    n, cf = 3000, 20.0
    res = np.zeros(n, np.float32)
    total_sent = np.zeros(n, np.float64)
    total_grad = np.zeros(n, np.float64)
    for it in range(30):
        g = workloads.normal_gradient(n, 1e-3, seed=50 + it)
        idx, val, _ = oracle.randomk_compress(g, res, [cf], seed=it)
        total_sent[idx] += val
        total_grad += g
    np.testing.assert_allclose(total_sent + res, total_grad, rtol=0, atol=1e-6)
