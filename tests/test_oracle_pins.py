"""Pins for the CPU oracle: every check here is independent of the oracle's own code.

The oracle is the full-sort definition of Top-k with error feedback and the
compression-gain statistic (Sec. II-C, Sec. III-B, Alg. 1 of the paper).  It is
checked against: the numbers the paper prints (kept fraction <-> CF), an O(n^2)
rank-counting brute force, numpy library routines (partition / sort / float32
add), closed forms, invariants and metamorphic relations.
"""
import math
import os

import numpy as np
import pytest

from oracle import oracle
from paper_2305_12201_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_rows(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def _mag(a):
    return a.view(np.uint32) & np.uint32(0x7FFFFFFF)


def brute_force_select(acc, k):
    """Rank-counting definition, independent of any sort:
    rank(i) = #{j : |a_j| > |a_i| or (|a_j| == |a_i| and j < i)}; selected <=> rank < k."""
    m = _mag(acc).astype(np.int64)
    n = m.size
    idx = np.arange(n)
    greater = m[None, :] > m[:, None]
    tie_before = (m[None, :] == m[:, None]) & (idx[None, :] < idx[:, None])
    rank = (greater | tie_before).sum(axis=1)
    return np.nonzero(rank < k)[0]


def run_oracle(grad, residual, cfs, commit=0, seg=None):
    res = residual.copy()
    idx, val, stats = oracle.compress(grad, res, cfs, commit, seg)
    return idx, val, stats, res


# --------------------------------------------------------------------------
# k from CF
# --------------------------------------------------------------------------

@pytest.mark.parametrize("name", ["cf_fraction.txt", "k_values.txt"])
def test_k_golden(name):
    for n, cf, k in _golden_rows(name):
        assert oracle.topk_count(int(n), float(cf)) == int(k)


def test_k_properties():
    assert oracle.topk_count(10, 1.5) == 7          # ceil(6.67)
    assert oracle.topk_count(3, 1000) == 1          # clamp to at least one
    assert oracle.topk_count(7, 1) == 7
    rng = np.random.default_rng(0)
    for _ in range(200):
        n = int(rng.integers(1, 10**9))
        a, b = int(rng.integers(1, 50)), int(rng.integers(1, 50))
        # nested ceilings: ceil(ceil(n/a)/b) == ceil(n/(ab))  (multi-level CF, Sec. IV-C)
        assert oracle.topk_count(oracle.topk_count(n, a), b) == oracle.topk_count(n, a * b)
        assert oracle.topk_count(n, a) == -(-n // a)


# --------------------------------------------------------------------------
# error-feedback add
# --------------------------------------------------------------------------

def test_accumulate_is_one_float32_add():
    rng = np.random.default_rng(1)
    n = 4096
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    r = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    # denormals must survive, and cancellation must give +0
    g[:4] = np.array([1e-40, -1e-40, 3e-39, 1.0], dtype=np.float32)
    r[:4] = np.array([1e-40, -1e-40, -3e-39, -1.0], dtype=np.float32)
    idx, val, stats, res = run_oracle(g, r, [1.0])
    acc = r + g                              # numpy float32 add: IEEE RNE, no flush
    assert np.array_equal(val.view(np.uint32), acc.view(np.uint32))
    assert val[0] != 0 and val[1] != 0       # 2e-40 is a denormal, not flushed
    assert val[2].view(np.uint32) == 0 and val[3].view(np.uint32) == 0   # x - x = +0
    assert np.array_equal(idx, np.arange(n, dtype=np.int32))
    assert math.isclose(stats[0, 0, 1], float((acc.astype(np.float64) ** 2).sum()), rel_tol=1e-12)


# --------------------------------------------------------------------------
# selection against brute force, with heavy ties and signed zeros
# --------------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(6))
def test_selection_matches_brute_force(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(5, 700))
    # quantised values force many equal magnitudes with mixed signs; plus exact zeros of both signs
    g = (rng.integers(-6, 7, n) * 0.125).astype(np.float32)
    r = (rng.integers(-2, 3, n) * 0.125).astype(np.float32)
    g[rng.random(n) < 0.1] = -0.0
    cf = float(rng.choice([1.0, 1.5, 2.0, 3.0, 7.0, 10.0, 1000.0]))
    k = -(-n // int(cf)) if cf == int(cf) else math.ceil(n / cf)
    idx, val, stats, res = run_oracle(g, r, [cf])
    acc = r + g
    expect = brute_force_select(acc, k)
    assert np.array_equal(idx, expect.astype(np.int32))
    assert np.array_equal(val.view(np.uint32), acc[expect].view(np.uint32))
    # residual: +0.0 on selected slots, acc (bit-identical, sign of -0 kept) elsewhere
    want = acc.copy()
    want[expect] = 0.0
    assert np.array_equal(res.view(np.uint32), want.view(np.uint32))
    # statistic from the brute-force set
    ss_sel = float((acc[expect].astype(np.float64) ** 2).sum())
    ss_all = float((acc.astype(np.float64) ** 2).sum())
    assert math.isclose(stats[0, 0, 0], ss_sel, rel_tol=1e-12, abs_tol=0)
    assert math.isclose(stats[0, 0, 1], ss_all, rel_tol=1e-12, abs_tol=0)
    if ss_all > 0:
        assert math.isclose(stats[0, 0, 2], ss_sel / ss_all, rel_tol=1e-12)


def test_ties_go_to_lower_index_and_zero_fill():
    # k exceeds the number of non-zeros: zero entries are taken by lowest index, still exactly k pairs
    g = np.zeros(16, dtype=np.float32)
    g[[3, 9]] = [2.0, -5.0]
    g[5] = -0.0
    idx, val, stats, res = run_oracle(g, np.zeros(16, np.float32), [4.0])   # k = 4
    assert idx.tolist() == [0, 1, 3, 9]
    assert val.tolist() == [0.0, 0.0, 2.0, -5.0]
    assert stats[0, 0, 3] == 0.0                       # smallest selected magnitude
    # all equal magnitudes with mixed signs: the first k positions win, signs are kept
    g = np.array([1, -1, 1, -1, 1, -1], dtype=np.float32)
    idx, val, _, res = run_oracle(g, np.zeros(6, np.float32), [2.0])
    assert idx.tolist() == [0, 1, 2] and val.tolist() == [1.0, -1.0, 1.0]
    assert res.tolist() == [0.0, 0.0, 0.0, -1.0, 1.0, -1.0]


def test_all_zero_gradient_has_gain_one():
    g = np.zeros(100, dtype=np.float32)
    idx, val, stats, res = run_oracle(g, g.copy(), [10.0])
    assert idx.tolist() == list(range(10))
    assert stats[0, 0].tolist() == [0.0, 0.0, 1.0, 0.0]


def test_nan_inf_order_by_bit_pattern():
    g = np.array([1.0, np.inf, -np.nan, 3.0, -np.inf, 2.0], dtype=np.float32)
    idx, val, stats, _ = run_oracle(g, np.zeros(6, np.float32), [2.0])   # k = 3
    assert idx.tolist() == [1, 2, 4]                  # NaN pattern above inf; inf tie -> lower index first
    assert np.isnan(stats[0, 0, 0])


# --------------------------------------------------------------------------
# library routines: numpy partition / sort on medium inputs
# --------------------------------------------------------------------------

@pytest.mark.parametrize("cf", [10.0, 100.0, 1000.0])
def test_threshold_and_multiset_match_numpy(cf):
    n = 300_000
    g = workloads.resnet_like_gradient(n, seed=5)
    r = workloads.normal_gradient(n, 1e-5, seed=6)
    idx, val, stats, res = run_oracle(g, r, [cf])
    acc = r + g
    k = -(-n // int(cf))
    assert idx.size == k
    mags = np.abs(acc)
    tau = np.partition(mags, n - k)[n - k]            # k-th largest magnitude, library routine
    assert stats[0, 0, 3] == float(tau)
    assert np.array_equal(np.sort(np.abs(val)), np.sort(mags)[n - k:])
    # invariants that fix the set uniquely
    assert np.all(np.diff(idx) > 0) and idx[0] >= 0 and idx[-1] < n
    sel = np.zeros(n, dtype=bool)
    sel[idx] = True
    assert mags[sel].min() >= mags[~sel].max()
    at_tau = np.nonzero(mags == tau)[0]
    taken = sel[at_tau]
    assert np.all(taken[:taken.sum()])                # among |acc| == tau the lowest indices are the taken ones
    # partition of acc into message and residual, bit for bit
    rebuilt = res.copy()
    rebuilt[idx] = val
    assert np.array_equal(rebuilt.view(np.uint32), acc.view(np.uint32))
    assert np.all(res[idx].view(np.uint32) == 0)
    # gain bounds (Sec. III-B: gain in (0, 1]); top-k mean square >= overall mean square
    gain = stats[0, 0, 2]
    assert k / n <= gain <= 1.0
    assert math.isclose(stats[0, 0, 0], float((val.astype(np.float64) ** 2).sum()), rel_tol=1e-12)


def test_cf_one_is_dense():
    n = 5000
    g = workloads.normal_gradient(n, 1e-3, seed=2)
    r = workloads.normal_gradient(n, 1e-4, seed=3)
    idx, val, stats, res = run_oracle(g, r, [1.0])
    assert np.array_equal(idx, np.arange(n, dtype=np.int32))
    assert np.array_equal(val, r + g)
    assert np.all(res.view(np.uint32) == 0)
    # dense SGD has gain 1.0 (Sec. III-B); numerator and denominator are summed in different orders
    assert math.isclose(stats[0, 0, 2], 1.0, rel_tol=1e-12)


# --------------------------------------------------------------------------
# several CFs in one call, commit semantics, nestedness, multi-level identity
# --------------------------------------------------------------------------

def test_multi_cf_stats_equal_single_cf_runs_and_nest():
    n = 200_000
    g = workloads.resnet_like_gradient(n, seed=11)
    r = workloads.normal_gradient(n, 1e-5, seed=12)
    cfs = [10.0, 100.0, 1000.0]
    singles = [run_oracle(g, r, [c]) for c in cfs]
    for commit in range(3):
        idx, val, stats, res = run_oracle(g, r, cfs, commit)
        assert np.array_equal(idx, singles[commit][0])
        assert np.array_equal(val.view(np.uint32), singles[commit][1].view(np.uint32))
        assert np.array_equal(res.view(np.uint32), singles[commit][3].view(np.uint32))
        for j in range(3):
            assert np.array_equal(stats[0, j], singles[j][2][0, 0])
    gains = [s[2][0, 0, 2] for s in singles]
    assert gains[0] > gains[1] > gains[2] > 0         # lower CF keeps more information (Sec. III-B)
    assert set(singles[2][0]) <= set(singles[1][0]) <= set(singles[0][0])


def test_multilevel_identity():
    """Sec. IV-C: C(theta2/theta1, C(theta1, X)) == C(theta2, X) for Top-k."""
    n = 123_457
    g = workloads.normal_gradient(n, 1e-3, seed=21)
    z = np.zeros(n, np.float32)
    i1, v1, _, _ = run_oracle(g, z, [10.0])
    i2, v2, _, _ = run_oracle(g, z, [1000.0])
    # second level: Top-k at CF 100 on the 10x message (positions in the message keep index order)
    j, w, _, _ = run_oracle(v1, np.zeros_like(v1), [100.0])
    assert np.array_equal(i1[j], i2)
    assert np.array_equal(w.view(np.uint32), v2.view(np.uint32))


def test_recompress_equals_direct_compression_and_moves_the_residual():
    """Sec. IV-C with the deferred commit: compress at theta1 and commit, recompress by theta2/theta1
    -> the same message, statistics and residual as compressing directly at theta2."""
    n = 40_003
    g = workloads.resnet_like_gradient(n, seed=23)
    r0 = workloads.normal_gradient(n, 1e-5, seed=24)
    for th1, rel in ((10.0, 100.0), (10.0, 10.0), (4.0, 2.5)):
        i1, v1, s1, res1 = run_oracle(g, r0, [th1])
        res = res1.copy()
        i2, v2, s2 = oracle.recompress(i1, v1, rel, residual=res)
        k2 = math.ceil(i1.size / rel)
        assert i2.size == k2
        # brute force on the message itself
        pos = brute_force_select(v1, k2)
        assert np.array_equal(i2, i1[pos]) and np.array_equal(v2.view(np.uint32), v1[pos].view(np.uint32))
        assert math.isclose(s2[0, 1], s1[0, 0, 0], rel_tol=1e-12)            # ||X1||^2
        assert math.isclose(s2[0, 0], float((v2.astype(np.float64) ** 2).sum()), rel_tol=1e-12)
        assert s2[0, 3] == float(np.abs(v2).min())
        if float(th1 * rel).is_integer() and math.ceil(math.ceil(n / th1) / rel) == math.ceil(n / (th1 * rel)):
            d_i, d_v, d_s, d_res = run_oracle(g, r0, [th1 * rel])
            assert np.array_equal(i2, d_i) and np.array_equal(v2.view(np.uint32), d_v.view(np.uint32))
            assert np.array_equal(res.view(np.uint32), d_res.view(np.uint32))
        # message + residual is still acc, bit for bit
        acc = r0 + g
        rebuilt = res.copy()
        rebuilt[i2] = v2
        assert np.array_equal(rebuilt.view(np.uint32), acc.view(np.uint32))
    # without a residual nothing else is touched; CF 1 keeps the whole message
    i2, v2, s2 = oracle.recompress(i1, v1, 1.0)
    assert np.array_equal(i2, i1) and np.array_equal(v2, v1) and math.isclose(s2[0, 2], 1.0, rel_tol=1e-12)


def test_recompress_layerwise():
    sizes = [64, 4096, 37, 100_003, 9408, 1000]
    off = workloads.offsets_of(sizes)
    n = int(off[-1])
    g = workloads.resnet_like_gradient(n, seed=25)
    z = np.zeros(n, np.float32)
    i1, v1, s1, res1 = run_oracle(g, z, [10.0], seg=off)
    counts = [-(-s // 10) for s in sizes]
    res = res1.copy()
    i2, v2, s2 = oracle.recompress(i1, v1, 10.0, residual=res, seg_counts=counts)
    d_i, d_v, d_s, d_res = run_oracle(g, z, [100.0], seg=off)
    assert np.array_equal(i2, d_i) and np.array_equal(v2.view(np.uint32), d_v.view(np.uint32))
    assert np.array_equal(res.view(np.uint32), d_res.view(np.uint32))
    assert np.allclose(s2[:, 0], d_s[:, 0, 0], rtol=1e-12) and np.array_equal(s2[:, 3], d_s[:, 0, 3])


def test_commit_takes_back_the_deferred_commit_and_dense_branch_rebuilds_acc():
    """The three branches of Alg. 1 after compress(theta_min) + recompress: candidate = as is; theta_min =
    commit of the level-1 indices gives the level-1 residual again; dense = residual + message is acc."""
    n = 60_001
    g = workloads.resnet_like_gradient(n, seed=27)
    r0 = workloads.normal_gradient(n, 1e-5, seed=28)
    i1, v1, _, res1 = run_oracle(g, r0, [10.0])
    res = res1.copy()
    i2, v2, _ = oracle.recompress(i1, v1, 8.0, residual=res)
    assert not np.array_equal(res.view(np.uint32), res1.view(np.uint32))
    back = res.copy()
    oracle.commit(i1, back)
    assert np.array_equal(back.view(np.uint32), res1.view(np.uint32))
    # against numpy's indexed assignment, with out-of-range indices skipped
    x = workloads.normal_gradient(1000, 1.0, seed=29)
    idx = np.array([5, -1, 999, 1000, 17, 5], np.int32)
    y = x.copy()
    oracle.commit(idx, y)
    z = x.copy()
    z[[5, 999, 17]] = 0.0
    assert np.array_equal(y.view(np.uint32), z.view(np.uint32)) and not np.signbit(y[[5, 999, 17]]).any()
    # dense branch: adding the level-2 message back into its residual restores acc exactly
    dense = res.copy()
    oracle.decompress_accumulate(i2, v2, [i2.size], dense)
    acc = r0 + g
    assert np.array_equal(dense.view(np.uint32), acc.view(np.uint32)) or \
        np.array_equal(np.where(acc == 0, 0.0, dense).view(np.uint32), np.where(acc == 0, 0.0, acc).view(np.uint32))


# --------------------------------------------------------------------------
# metamorphic relations
# --------------------------------------------------------------------------

def test_scaling_sign_flip_and_permutation():
    n = 50_000
    g = workloads.resnet_like_gradient(n, seed=31)
    r = workloads.normal_gradient(n, 1e-5, seed=32)
    cfs = [10.0, 100.0]
    i0, v0, s0, _ = run_oracle(g, r, cfs)
    # power-of-two scaling is exact in binary32 (no overflow/underflow here): same indices and gain
    i1, v1, s1, _ = run_oracle(g * np.float32(8), r * np.float32(8), cfs)
    assert np.array_equal(i0, i1) and np.array_equal(v1, v0 * np.float32(8))
    assert np.allclose(s1[0, :, 2], s0[0, :, 2], rtol=1e-13)
    assert np.allclose(s1[0, :, 0], 64 * s0[0, :, 0], rtol=1e-13)
    # flipping every sign: same indices, negated values, same statistics
    i2, v2, s2, _ = run_oracle(-g, -r, cfs)
    assert np.array_equal(i0, i2) and np.array_equal(v2, -v0)
    assert np.array_equal(s2, s0)
    # permuting the elements leaves the statistics unchanged (up to summation order)
    p = np.random.default_rng(3).permutation(n)
    _, _, s3, _ = run_oracle(g[p].copy(), r[p].copy(), cfs)
    assert np.allclose(s3, s0, rtol=1e-12)


# --------------------------------------------------------------------------
# closed forms for the gain
# --------------------------------------------------------------------------

def test_gain_closed_form_permutation_of_integers():
    n, cf = 4000, 8.0
    k = 500
    vals = np.random.default_rng(4).permutation(np.arange(1, n + 1)).astype(np.float32)
    signs = np.where(np.random.default_rng(5).random(n) < 0.5, -1, 1).astype(np.float32)
    idx, val, stats, _ = run_oracle(vals * signs, np.zeros(n, np.float32), [cf])

    def sum_sq(m):                                    # 1^2 + ... + m^2
        return m * (m + 1) * (2 * m + 1) // 6

    assert stats[0, 0, 0] == float(sum_sq(n) - sum_sq(n - k))
    assert stats[0, 0, 1] == float(sum_sq(n))
    assert stats[0, 0, 3] == float(n - k + 1)
    assert sorted(np.abs(val).tolist()) == list(range(n - k + 1, n + 1))


def test_gain_asymptotics_normal_and_laplace():
    """Large-n sanity against the analytic tail energy of the distribution."""
    from scipy.stats import norm
    n, p = 2_000_000, 0.01
    z = np.zeros(n, np.float32)
    t = norm.ppf(1 - p / 2)
    want_normal = p + 2 * t * norm.pdf(t)             # E[x^2; |x|>t] for a unit normal
    _, _, s, _ = run_oracle(workloads.normal_gradient(n, 1e-3, seed=41), z, [100.0])
    assert abs(s[0, 0, 2] - want_normal) / want_normal < 0.02
    L = math.log(1 / p)
    want_laplace = p * (L * L + 2 * L + 2) / 2        # tail energy of a unit-scale Laplace over its variance 2
    _, _, s, _ = run_oracle(workloads.resnet_like_gradient(n, seed=42, outlier_frac=0.0), z, [100.0])
    assert abs(s[0, 0, 2] - want_laplace) / want_laplace < 0.02


# --------------------------------------------------------------------------
# error feedback over iterations: nothing is ever dropped
# --------------------------------------------------------------------------

def test_error_feedback_conserves_the_gradient_sum():
    n, iters = 20_000, 6
    res = np.zeros(n, np.float32)
    sent = np.zeros(n, np.float64)
    total = np.zeros(n, np.float64)
    prev_leftover_hit = False
    for it in range(iters):
        g = workloads.normal_gradient(n, 1e-3, seed=50 + it)
        before = res.copy()
        idx, val, _ = oracle.compress(g, res, [100.0])
        sent[idx] += val.astype(np.float64)
        total += g.astype(np.float64)
        if it > 0:
            # entries that carried a large leftover are more likely to be chosen now
            prev_leftover_hit |= bool(np.abs(before[idx]).mean() > np.abs(before).mean())
    assert np.allclose(sent + res, total, rtol=0, atol=iters * 2e-10)
    assert prev_leftover_hit


# --------------------------------------------------------------------------
# layerwise (segmented) mode
# --------------------------------------------------------------------------

def test_segmented_equals_independent_runs_with_global_indices():
    sizes = [64, 1, 4096, 37, 100_003, 2, 9408, 64, 64, 1000]
    off = workloads.offsets_of(sizes)
    n = int(off[-1])
    g = workloads.resnet_like_gradient(n, seed=61)
    r = workloads.normal_gradient(n, 1e-5, seed=62)
    cfs = [100.0, 10.0]
    idx, val, stats, res = run_oracle(g, r, cfs, commit=0, seg=off)
    at = 0
    for t, s in enumerate(sizes):
        a, b = int(off[t]), int(off[t + 1])
        i_t, v_t, s_t, r_t = run_oracle(g[a:b].copy(), r[a:b].copy(), cfs, 0)
        k = i_t.size
        assert k == -(-s // 100)
        assert np.array_equal(idx[at:at + k], i_t + a)
        assert np.array_equal(val[at:at + k], v_t)
        assert np.array_equal(res[a:b], r_t)
        assert np.array_equal(stats[t], s_t[0])
        at += k
    assert at == idx.size


# --------------------------------------------------------------------------
# decompression
# --------------------------------------------------------------------------

def test_decompress_accumulate_definition():
    rng = np.random.default_rng(7)
    n, W = 1000, 5
    idxs, vals, counts = [], [], []
    dense = rng.standard_normal(n).astype(np.float32)
    want = dense.copy()
    for w in range(W):
        k = int(rng.integers(0, 200))
        i = np.sort(rng.choice(n, size=k, replace=False)).astype(np.int32)
        v = rng.standard_normal(k).astype(np.float32)
        idxs.append(i), vals.append(v), counts.append(k)
        for a, b in zip(i.tolist(), v.tolist()):      # the double loop, float32 adds in worker order
            want[a] = np.float32(want[a] + np.float32(b))
    oracle.decompress_accumulate(np.concatenate(idxs), np.concatenate(vals), counts, dense)
    assert np.array_equal(dense.view(np.uint32), want.view(np.uint32))


def test_decompress_inverts_compress():
    n = 10_000
    g = workloads.normal_gradient(n, 1e-3, seed=71)
    idx, val, _, res = run_oracle(g, np.zeros(n, np.float32), [1.0])
    dense = np.zeros(n, np.float32)
    oracle.decompress_accumulate(idx, val, [idx.size], dense)
    assert np.array_equal(dense, g)                   # CF 1 message rebuilds acc
    idx, val, _, res = run_oracle(g, np.zeros(n, np.float32), [50.0])
    dense = np.zeros(n, np.float32)
    oracle.decompress_accumulate(idx, val, [idx.size], dense)
    assert np.array_equal(dense + res, g)             # message + residual = acc


def test_decompress_update_hand_values():
    """Alg. 1's update w - eta * aggregate, taken pair by pair: values worked out by hand."""
    # exact binary fractions: w = [1, 2, 3, 4], two workers, alpha = -1/4 (eta = 0.5, W = 2)
    w = np.array([1.0, 2.0, 3.0, 4.0], np.float32)
    oracle.decompress_update(np.array([0, 2, 2, 3], np.int32), np.array([4.0, 8.0, -2.0, 1.0], np.float32), [2, 2], -0.25, w)
    assert w.tolist() == [0.0, 2.0, 1.5, 3.75]
    # the product is rounded before the sum: (1 + 2^-12)^2 = 1 + 2^-11 + 2^-24 rounds to 1 + 2^-11 (a tie, to the even
    # mantissa), and w = -(1 + 2^-11) then gives exactly 0; a fused multiply-add would leave 2^-24
    a = np.float32(1.0 + 2.0 ** -12)
    w = np.array([-(1.0 + 2.0 ** -11)], np.float32)
    oracle.decompress_update(np.array([0], np.int32), np.array([a], np.float32), [1], float(a), w)
    assert w[0] == 0.0
    # workers in order: (2^24 + 1) + 1 = 2^24 + 2 needs two adds of 1 to be taken one by one ... and both are lost
    # (2^24 + 1 is not a binary32 number, ties to even), while one add of 2 is not
    w = np.array([2.0 ** 24, 2.0 ** 24], np.float32)
    oracle.decompress_update(np.array([0, 1, 0], np.int32), np.array([1.0, 2.0, 1.0], np.float32), [2, 1], 1.0, w)
    assert w.tolist() == [2.0 ** 24, 2.0 ** 24 + 2.0]
    # order matters: big, then -big, then small keeps the small one; small first loses it
    w = np.zeros(2, np.float32)
    oracle.decompress_update(np.array([0, 1, 0, 1, 0, 1], np.int32),
                             np.array([1e8, 1.0, -1e8, 1e8, 1.0, -1e8], np.float32), [2, 2, 2], 1.0, w)
    assert w.tolist() == [1.0, 0.0]


def test_decompress_update_against_library_arithmetic():
    rng = np.random.default_rng(19)
    n, W = 3000, 6
    w0 = rng.standard_normal(n).astype(np.float32)
    idxs, vals, counts = [], [], []
    for _ in range(W):
        k = int(rng.integers(0, 900))
        idxs.append(np.sort(rng.choice(n, size=k, replace=False)).astype(np.int32))
        vals.append((rng.standard_normal(k) * 1e-2).astype(np.float32))
        counts.append(k)
    idx, val = np.concatenate(idxs), np.concatenate(vals)
    alpha = np.float32(-0.1 / W)
    # numpy's float32 arithmetic, one worker at a time (indices within a worker are distinct, so fancy indexing is safe)
    want = w0.copy()
    for i, v in zip(idxs, vals):
        want[i] = want[i] + alpha * v
    got = w0.copy()
    oracle.decompress_update(idx, val, counts, float(alpha), got)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # against the definition in exact arithmetic: w - eta * mean of the decompressed messages, within W + 1 roundings
    dense = np.zeros(n, np.float64)
    for i, v in zip(idxs, vals):
        dense[i] += v.astype(np.float64)
    exact = w0.astype(np.float64) - 0.1 * dense / W
    tol = (2 * W + 2) * 2.0 ** -24 * (np.abs(w0.astype(np.float64)) + 0.1 * np.abs(dense) + 1e-3)
    assert np.all(np.abs(got.astype(np.float64) - exact) <= tol)
    # alpha = 1 is the plain accumulation
    a, b = w0.copy(), w0.copy()
    oracle.decompress_update(idx, val, counts, 1.0, a)
    oracle.decompress_accumulate(idx, val, counts, b)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    # entries no pair names stay as they are, bit for bit
    untouched = np.setdiff1d(np.arange(n), idx)
    assert np.array_equal(got[untouched].view(np.uint32), w0[untouched].view(np.uint32))


def test_decompress_update_rejects_bad_arguments():
    w = np.zeros(4, np.float32)
    with pytest.raises(RuntimeError):
        oracle.decompress_update(np.array([4], np.int32), np.array([1.0], np.float32), [1], 1.0, w)
    with pytest.raises(RuntimeError):
        oracle.decompress_update(np.array([0], np.int32), np.array([1.0], np.float32), [-1], 1.0, w)


# --------------------------------------------------------------------------
# workload shapes
# --------------------------------------------------------------------------

def test_workload_shapes():
    rs = workloads.resnet101_tensor_sizes()
    assert len(rs) == 314 and sum(rs) == 44_549_160 and min(rs) == 64 and max(rs) == 2_359_296
    assert sum(-(-s // 100) for s in rs) == 445_667
    vs = workloads.vgg16_tensor_sizes()
    assert sum(vs) == 138_357_544 and sum(vs[:26]) == 14_714_688 and sum(vs[26:]) == 123_642_856
    assert sum(workloads.lstm_tensor_sizes()) == 50_065_078
    g = workloads.lstm_like_gradient(0, vocab=2000, hidden=50)
    emb = g[:2000 * 50].reshape(2000, 50)
    zero_rows = int((np.abs(emb).sum(axis=1) == 0).sum())
    assert zero_rows == 1900
