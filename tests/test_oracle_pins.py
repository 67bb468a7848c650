"""Pins for the CPU oracle: values and properties fixed by the paper and by the
mathematics, none of them produced by the oracle itself or by the GPU path.

Each test is chosen so that one plausible mistake in oracle/kb_oracle.c (dropped
term, wrong sign or index, transposed operand, wrong tie rule) fails it.
"""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
from paper_2511_18868_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _one(n, k):
    return np.array([0, n], np.int32), np.array([0, k], np.int32)


# ------------------------------------------------------------------ prune

def test_bound_hand_values():
    # golden/roofline_hand.txt: values worked by hand from the roofline model
    # (Assumption 1): runtime >= max(flops/peak_flops, bytes/peak_bw)
    rows = [l.split() for l in open(os.path.join(GOLD, "roofline_hand.txt"))
            if l.strip() and not l.startswith("#")]
    flops = np.array([float(r[0]) for r in rows], np.float32)
    byts = np.array([float(r[1]) for r in rows], np.float32)
    want = np.array([float(r[2]) for r in rows])
    seg, _ = _one(len(rows), 1)
    bound, alive = oracle.prune(seg, flops, byts, 2.5e15, 8e12, np.array([2e-3], np.float32))
    np.testing.assert_allclose(bound, want, rtol=2e-7)
    # rows far from the incumbent on either side
    want_alive = np.array([int(r[3]) for r in rows], np.uint8)
    np.testing.assert_array_equal(alive, want_alive)


def test_bound_machine_balance_crossover():
    # below 312.5 flop/B the memory term wins, above it the compute term
    byts = np.full(3, 1e9, np.float32)
    flops = np.array([1e9 * 100.0, 1e9 * 312.5, 1e9 * 1000.0], np.float32)
    seg, _ = _one(3, 1)
    bound, _ = oracle.prune(seg, flops, byts, 2.5e15, 8e12, np.array([np.inf], np.float32))
    mem = np.float32(1e9) / np.float32(8e12)
    np.testing.assert_array_equal(bound[0], mem)
    np.testing.assert_allclose(bound[1], float(mem), rtol=2e-7)
    np.testing.assert_array_equal(bound[2], np.float32(1e12) / np.float32(2.5e15))


def test_mask_invariants_and_extremes():
    b = synth.config3(G=7, Ng=101)
    bound, alive = oracle.prune(b.seg_off, b.flops, b.bytes_, b.peak_flops, b.peak_bw, b.incumbent)
    for g in range(b.G):
        sl = slice(b.seg_off[g], b.seg_off[g + 1])
        assert np.all(bound[sl][alive[sl] == 0] >= b.incumbent[g])
        assert np.all(bound[sl][alive[sl] == 1] < b.incumbent[g])
        # distinct bounds + lower-median incumbent: exactly floor((n-1)/2) alive,
        # and the equality branch is exercised (incumbent is one of the bounds)
        assert len(np.unique(bound[sl])) == 101
        assert alive[sl].sum() == (101 - 1) // 2
        assert np.any(bound[sl] == b.incumbent[g])
    _, all_alive = oracle.prune(b.seg_off, b.flops, b.bytes_, b.peak_flops, b.peak_bw,
                                np.full(b.G, np.inf, np.float32))
    assert all_alive.all()
    _, none_alive = oracle.prune(b.seg_off, b.flops, b.bytes_, b.peak_flops, b.peak_bw,
                                 np.zeros(b.G, np.float32))
    assert not none_alive.any()


def test_mask_scale_invariance():
    # doubling flops, bytes and the incumbent is exact in binary floating point
    b = synth.config1()
    _, a1 = oracle.prune(b.seg_off, b.flops, b.bytes_, b.peak_flops, b.peak_bw, b.incumbent)
    bd2, a2 = oracle.prune(b.seg_off, 2 * b.flops, 2 * b.bytes_, b.peak_flops, b.peak_bw,
                           2 * b.incumbent)
    np.testing.assert_array_equal(a1, a2)
    bd1, _ = oracle.prune(b.seg_off, b.flops, b.bytes_, b.peak_flops, b.peak_bw, b.incumbent)
    np.testing.assert_array_equal(bd2, 2 * bd1)


def test_bound_is_fp32_division():
    # numpy's float32 division is IEEE RNE; the oracle must round the same way
    rng = np.random.default_rng(1)
    flops = (10 ** rng.uniform(6, 12, 5000)).astype(np.float32)
    byts = (10 ** rng.uniform(6, 12, 5000)).astype(np.float32)
    seg, _ = _one(5000, 1)
    bound, _ = oracle.prune(seg, flops, byts, 2.5e15, 8e12, np.array([1.0], np.float32))
    want = np.maximum(flops / np.float32(2.5e15), byts / np.float32(8e12))
    np.testing.assert_array_equal(bound, want)


# ------------------------------------------------------------- Lloyd step

def test_k1_closed_form():
    # K = 1: the centroid is the column mean, and on z-scored (ddof = 0) data
    # J = N*D once the centroid is the mean
    b = synth.config2(N=500, D=12, K=1)
    r1 = oracle.cluster_step(b.seg_off, b.koff, b.X, b.X[:1])
    np.testing.assert_allclose(r1.cent[0], b.X.astype(np.float64).mean(axis=0), atol=1e-7)
    assert r1.counts[0] == 500 and not r1.flag.any() and (r1.assign == 0).all()
    r2 = oracle.cluster_step(b.seg_off, b.koff, b.X, r1.cent)
    assert abs(r2.objective[0] - 500 * 12) < 1e-3


def test_k_equals_n_identity():
    b = synth.config1(N=40, D=6, K=40)
    r = oracle.cluster_step(b.seg_off, b.koff, b.X, b.X[:40])
    np.testing.assert_array_equal(r.assign, np.arange(40))
    assert r.objective[0] == 0.0
    np.testing.assert_array_equal(r.cent, b.X)
    np.testing.assert_array_equal(r.counts, np.ones(40, np.int32))


def test_step_equals_pairwise_matrix_and_groupby():
    # one step = argmin over the pairwise squared-distance matrix + group-by mean
    b = synth.config3(G=3, Ng=200, D=7, K=5)
    cin = synth.random_centroids(b, 3)
    r = oracle.cluster_step(b.seg_off, b.koff, b.X, cin)
    for g in range(b.G):
        x = b.X[b.seg_off[g]:b.seg_off[g + 1]].astype(np.float64)
        c = cin[b.koff[g]:b.koff[g + 1]].astype(np.float64)
        d2 = ((x[:, None, :] - c[None, :, :]) ** 2).sum(-1)
        a = d2.argmin(1)
        np.testing.assert_array_equal(r.assign[b.seg_off[g]:b.seg_off[g + 1]], a)
        np.testing.assert_allclose(r.objective[g], d2.min(1).sum(), rtol=1e-12)
        for j in range(5):
            np.testing.assert_allclose(r.cent[b.koff[g] + j], x[a == j].mean(0), rtol=0, atol=1e-6)
            assert r.counts[b.koff[g] + j] == (a == j).sum()


def test_step_vs_sklearn_single_iteration():
    sk = pytest.importorskip("sklearn.cluster")
    b = synth.config2(N=600, D=9, K=6)
    cin = synth.random_centroids(b, 11)
    r = oracle.cluster_step(b.seg_off, b.koff, b.X, cin)
    assert (r.counts > 0).all()
    km = sk.KMeans(n_clusters=6, init=cin.astype(np.float64), n_init=1, max_iter=1,
                   algorithm="lloyd", tol=0.0).fit(b.X.astype(np.float64))
    np.testing.assert_allclose(km.cluster_centers_, r.cent, atol=1e-5)


def _brute_force_opt(x, K):
    n = len(x)
    best = np.inf
    best_lab = None
    for lab in itertools.product(range(K), repeat=n):
        lab = np.array(lab)
        J = 0.0
        for j in range(K):
            m = x[lab == j]
            if len(m):
                J += ((m - m.mean(0)) ** 2).sum()
        if J < best - 1e-12:
            best, best_lab = J, lab
    return best, best_lab


def test_lloyd_vs_bruteforce_optimum():
    rng = np.random.default_rng(5)
    # well-separated blobs: Lloyd from the first K rows reaches the optimum
    cent = np.array([[0, 0], [10, 0], [0, 10]], float)
    x = np.concatenate([cent, cent[rng.integers(0, 3, 6)]]) + 0.3 * rng.standard_normal((9, 2))
    x = x.astype(np.float32)
    seg, ko = _one(9, 3)
    r = oracle.cluster(seg, ko, x, 10)
    Jopt, lab = _brute_force_opt(x.astype(np.float64), 3)
    # objective reported is relative to centroids entering the last step, which
    # at a fixed point are the cluster means
    assert abs(r.objective[0] - Jopt) < 1e-9
    # same partition (labels may be permuted)
    assert len({(a, l) for a, l in zip(r.assign, lab)}) == 3
    # random clouds: J_opt <= J_Lloyd always
    for seed in range(4):
        x = np.random.default_rng(seed).standard_normal((8, 2)).astype(np.float32)
        seg, ko = _one(8, 2)
        r = oracle.cluster(seg, ko, x, 12)
        Jopt, _ = _brute_force_opt(x.astype(np.float64), 2)
        assert Jopt <= r.objective[0] + 1e-9


def _dp_1d_opt(x, K):
    xs = np.sort(x)
    n = len(xs)
    cost = np.zeros((n + 1, n + 1))
    for i in range(n):
        for j in range(i + 1, n + 1):
            m = xs[i:j]
            cost[i, j] = ((m - m.mean()) ** 2).sum()
    dp = np.full((K + 1, n + 1), np.inf)
    dp[0, 0] = 0
    for k in range(1, K + 1):
        for j in range(1, n + 1):
            for i in range(k - 1, j):
                dp[k, j] = min(dp[k, j], dp[k - 1, i] + cost[i, j])
    return dp[K, n]


def test_1d_interval_dp_lower_bound():
    for seed in range(3):
        x = np.random.default_rng(100 + seed).standard_normal(30).astype(np.float32)
        seg, ko = _one(30, 3)
        r = oracle.cluster(seg, ko, x[:, None], 25)
        assert _dp_1d_opt(x.astype(np.float64), 3) <= r.objective[0] + 1e-9


def test_lloyd_invariants():
    b = synth.config5(G=12, nmin=64, nmax=400)
    cur = np.concatenate([b.X[b.seg_off[g]:b.seg_off[g] + (b.koff[g + 1] - b.koff[g])]
                          for g in range(b.G)])
    prevJ = np.full(b.G, np.inf)
    for it in range(8):
        r = oracle.cluster_step(b.seg_off, b.koff, b.X, cur)
        assert np.all(r.objective <= prevJ * (1 + 1e-12))          # non-increasing
        prevJ = r.objective
        for g in range(b.G):
            a = r.assign[b.seg_off[g]:b.seg_off[g + 1]]
            x = b.X[b.seg_off[g]:b.seg_off[g + 1]].astype(np.float64)
            K = b.koff[g + 1] - b.koff[g]
            cnt = r.counts[b.koff[g]:b.koff[g + 1]]
            assert cnt.sum() == len(a)                              # sizes sum to N_g
            np.testing.assert_array_equal(cnt, np.bincount(a, minlength=K))
            c = cur[b.koff[g]:b.koff[g + 1]].astype(np.float64)
            d2 = ((x[:, None] - c[None]) ** 2).sum(-1)
            own = d2[np.arange(len(a)), a]
            assert np.all(own[:, None] <= d2 + 1e-12)               # nearest centroid
            for j in range(K):
                if cnt[j]:
                    np.testing.assert_allclose(r.cent[b.koff[g] + j], x[a == j].mean(0), atol=1e-6)
        cur = r.cent
    # cluster() == iterated cluster_step()
    full = oracle.cluster(b.seg_off, b.koff, b.X, 8)
    np.testing.assert_array_equal(full.assign, r.assign)
    np.testing.assert_array_equal(full.cent, r.cent)
    np.testing.assert_array_equal(full.counts, r.counts)
    np.testing.assert_array_equal(full.objective, r.objective)


def test_converged_step_is_idempotent():
    b = synth.config2(N=300, D=4, K=3)
    r = oracle.cluster(b.seg_off, b.koff, b.X, 60)
    r2 = oracle.cluster_step(b.seg_off, b.koff, b.X, r.cent)
    np.testing.assert_array_equal(r2.assign, r.assign)
    np.testing.assert_array_equal(r2.cent, r.cent)


def test_translation_invariance():
    b = synth.config2(N=400, D=8, K=7)
    cin = synth.random_centroids(b, 2)
    r = oracle.cluster_step(b.seg_off, b.koff, b.X, cin)
    shift = np.float32(4.0)   # power of two keeps the shifted fp32 inputs close to exact
    r2 = oracle.cluster_step(b.seg_off, b.koff, b.X + shift, cin + shift)
    ok = r.flag == 0
    np.testing.assert_array_equal(r.assign[ok], r2.assign[ok])


def test_tie_breaks_lowest_index():
    x = np.array([[0, 0], [2, 0], [1, 0], [1, 5], [-3, 1]], np.float32)
    seg, ko = _one(5, 3)
    # duplicate centroids 0 and 1: everything nearer to them goes to index 0
    cin = np.array([[1, 0], [1, 0], [50, 50]], np.float32)
    r = oracle.cluster_step(seg, ko, x, cin)
    np.testing.assert_array_equal(r.assign, np.zeros(5, np.int32))
    assert r.flag.all()
    # points at exactly equal (integer) distance from centroids 1 and 2 -> 1
    cin = np.array([[100, 100], [0, 0], [2, 0]], np.float32)
    r = oracle.cluster_step(seg, ko, x, cin)
    np.testing.assert_array_equal(r.assign, [1, 2, 1, 1, 1])
    np.testing.assert_array_equal(r.flag, [0, 0, 1, 1, 0])


def test_near_tie_flag_threshold():
    # 1-D: centroids at 0 and 2; x = 1 + e has d1 = (1+e)^2, d2 = (1-e)^2,
    # relative gap ~ 4e.  e = 0 (an exact tie) flags, e = 1e-3 does not.  (Where the
    # threshold lies in between is pinned in test_oracle_pins_flags.py.)
    seg, ko = _one(2, 2)
    cin = np.array([[0.0], [2.0]], np.float32)
    x = np.array([[1.0 + 1e-3], [1.0]], np.float32)
    r = oracle.cluster_step(seg, ko, x, cin)
    np.testing.assert_array_equal(r.flag, [0, 1])
    np.testing.assert_array_equal(r.assign, [1, 0])


def test_empty_cluster_keeps_centroid():
    b = synth.config1(N=64, D=4, K=4)
    X = b.X.copy()
    X[1] = X[0]
    # first step from the first K rows: rows 0 and 1 coincide, so every point
    # that is nearest to that location goes to cluster 0 and cluster 1 is empty;
    # its centroid must come out unchanged
    r = oracle.cluster(b.seg_off, b.koff, X, 1)
    assert r.counts[1] == 0
    np.testing.assert_array_equal(r.cent[1], X[0])
    assert r.counts.sum() == 64
    assert r.counts[0] >= 2 and r.assign[0] == 0 and r.assign[1] == 0
    # a centroid no point is nearest to stays put for good
    cin = np.concatenate([b.X[:3], np.full((1, 4), 1e3, np.float32)])
    r = oracle.cluster(b.seg_off, b.koff, b.X, 5, cent_init=cin)
    assert r.counts[3] == 0
    np.testing.assert_array_equal(r.cent[3], cin[3])


def test_cluster_iters0_and_cent_init():
    b = synth.config1(N=64, D=4, K=4)
    r = oracle.cluster(b.seg_off, b.koff, b.X, 0)
    np.testing.assert_array_equal(r.cent, b.X[:4])
    assert (r.assign == -1).all()
    cin = synth.random_centroids(b, 9)
    r1 = oracle.cluster(b.seg_off, b.koff, b.X, 1, cent_init=cin)
    s1 = oracle.cluster_step(b.seg_off, b.koff, b.X, cin)
    np.testing.assert_array_equal(r1.assign, s1.assign)
    np.testing.assert_array_equal(r1.cent, s1.cent)


# -------------------------------------------------------------------- UCB

def _ucb_single(K, S, assign, alive, bound, visits, rsum, t, c, pn=0.0, pm=0.5):
    n = len(assign)
    seg, ko = _one(n, K)
    return oracle.ucb_select(seg, ko, S, np.asarray(assign, np.int32), np.asarray(alive, np.uint8),
                             np.asarray(bound, np.float32), np.asarray(visits, np.int32),
                             np.asarray(rsum, np.float32), np.array([t], np.int64), c, pn, pm)


def test_ucb_initial_state_of_algorithm_1():
    # N = 1, mu = 0.5 for every arm and t = 1 (ln t = 0): every score is 0.5,
    # the argmax is an all-way tie, resolved to the lowest index (0, 0)
    K, S, n = 3, 6, 7
    r = _ucb_single(K, S, [0, 1, 2, 0, 1, 2, 0], np.ones(n), np.arange(n, 0, -1) * 1e-3,
                    np.zeros((n, S)), np.zeros((n, S)), 1, 2.0, pn=1.0, pm=0.5)
    np.testing.assert_array_equal(r.ucb, np.full((K, S), 0.5))
    np.testing.assert_array_equal(r.mu, np.full((K, S), 0.5))
    assert tuple(r.sel[0][:2]) == (0, 0)
    assert r.sel[0][2] == 6          # cluster 0 = {0, 3, 6}; candidate 6 has the smallest bound
    assert r.near[0] == 0


def test_ucb_hand_value():
    # golden/ucb_hand.txt: mu = 0.25, N = 4, t = 55, c = 2
    #   0.25 + 2*sqrt(ln 55 / 4) = 0.25 + sqrt(ln 55)
    want = [float(l) for l in open(os.path.join(GOLD, "ucb_hand.txt"))
            if l.strip() and not l.startswith("#")][0]
    assert abs(want - (0.25 + math.sqrt(math.log(55.0)))) < 5e-7
    r = _ucb_single(1, 1, [0, 0], [1, 1], [1.0, 2.0], [[3], [1]], [[1.0], [0.0]], 55, 2.0)
    assert r.Ncs[0, 0] == 4
    assert abs(r.mu[0, 0] - 0.25) < 1e-15
    assert abs(r.ucb[0, 0] - want) < 5e-7


def test_ucb_monotonicity_and_range():
    # score decreases in N at fixed mu, increases in t; mu in [0, 1]
    prev = np.inf
    for n in [1, 2, 5, 50, 500]:
        r = _ucb_single(1, 1, [0], [1], [1.0], [[2 * n]], [[n]], 1000, 1.3)
        assert abs(r.mu[0, 0] - 0.5) < 1e-15
        assert r.ucb[0, 0] < prev
        prev = r.ucb[0, 0]
    prev = -np.inf
    for t in [1, 2, 10, 10 ** 6, 10 ** 12]:
        r = _ucb_single(1, 1, [0], [1], [1.0], [[4]], [[1]], t, 1.3)
        assert r.ucb[0, 0] > prev
        prev = r.ucb[0, 0]
    b = synth.config1()
    o = oracle.round_(b)
    ok = np.isfinite(o.mu)
    assert np.all(o.mu[ok] >= 0) and np.all(o.mu[ok] <= 1)


def test_running_mean_identity():
    # Alg. 1's update mu += (r - mu)/N from (N, mu) = (1, 0.5) ends at
    # (prior_n*prior_mu + sum r) / (prior_n + n), which is what the oracle forms
    rng = np.random.default_rng(3)
    rewards = rng.random(37)
    N, mu = 1, 0.5
    for r_ in rewards:
        N += 1
        mu += (r_ - mu) / N
    r = _ucb_single(1, 1, [0], [1], [1.0], [[37]], [[np.float32(0)]], 5, 2.0, pn=1.0, pm=0.5)
    assert r.Ncs[0, 0] == 37
    # feed the rewards as 37 members with one visit each so the sum is formed by the oracle
    r = _ucb_single(1, 1, [0] * 37, [1] * 37, np.ones(37), np.ones((37, 1)),
                    rewards.astype(np.float32)[:, None], 5, 2.0, pn=1.0, pm=0.5)
    want = (0.5 + rewards.astype(np.float32).astype(np.float64).sum()) / 38
    assert abs(r.mu[0, 0] - want) < 1e-14
    assert abs(r.mu[0, 0] - mu) < 1e-7


def test_ucb_untried_arm_and_masked_cluster():
    K, S = 3, 2
    assign = [0, 0, 1, 1, 2]
    alive = [1, 1, 0, 0, 1]                 # cluster 1 has no alive member
    visits = [[3, 2], [1, 1], [9, 9], [9, 9], [0, 4]]
    rsum = [[1, 1], [0, 1], [9, 9], [9, 9], [0, 2]]
    r = _ucb_single(K, S, assign, alive, [5., 4., 1., 1., 3.], visits, rsum, 30, 1.0)
    assert np.all(np.isneginf(r.ucb[1]))
    assert np.isposinf(r.ucb[2, 0]) and np.isnan(r.mu[2, 0])
    np.testing.assert_array_equal(r.Ncs, [[4, 3], [0, 0], [0, 4]])
    np.testing.assert_array_equal(r.sel[0], [2, 0, 4])
    # nothing alive at all
    r = _ucb_single(K, S, assign, [0] * 5, [5., 4., 1., 1., 3.], visits, rsum, 30, 1.0)
    np.testing.assert_array_equal(r.sel[0], [-1, -1, -1])


def test_selection_bruteforce():
    b = synth.config5(G=20, nmin=64, nmax=300, S=5)
    bound, alive = oracle.prune(b.seg_off, b.flops, b.bytes_, b.peak_flops, b.peak_bw, b.incumbent)
    cl = oracle.cluster(b.seg_off, b.koff, b.X, 5)
    r = oracle.ucb_select(b.seg_off, b.koff, b.S, cl.assign, alive, bound, b.visits, b.rsum,
                          b.t, b.c)
    for g in range(b.G):
        sl = slice(b.seg_off[g], b.seg_off[g + 1])
        K = b.koff[g + 1] - b.koff[g]
        a, al = cl.assign[sl], alive[sl].astype(bool)
        best, arg = -np.inf, None
        for i in range(K):
            m = (a == i) & al
            if not m.any():
                assert np.all(np.isneginf(r.ucb[b.koff[g] + i]))
                continue
            for s in range(b.S):
                n = b.visits[sl][m, s].sum()
                R = b.rsum[sl][m, s].astype(np.float64).sum()
                assert r.Ncs[b.koff[g] + i, s] == n
                u = R / n + b.c * math.sqrt(math.log(b.t[g]) / n)
                assert abs(u - r.ucb[b.koff[g] + i, s]) < 1e-12
                if u > best:
                    best, arg = u, (i, s)
        I, Ss, ks = r.sel[g]
        if not r.near[g]:
            assert (I, Ss) == arg
        kl = ks - b.seg_off[g]
        assert al[kl] and a[kl] == I
        members = np.where((a == I) & al)[0]
        assert bound[sl][kl] == bound[sl][members].min()
        assert kl == members[np.argmin(bound[sl][members])]


def test_forcing_the_cluster_by_masking():
    b = synth.config1()
    bound, _ = oracle.prune(b.seg_off, b.flops, b.bytes_, b.peak_flops, b.peak_bw, b.incumbent)
    cl = oracle.cluster(b.seg_off, b.koff, b.X, 5)
    for target in range(8):
        alive = (cl.assign == target).astype(np.uint8)
        r = oracle.ucb_select(b.seg_off, b.koff, b.S, cl.assign, alive, bound, b.visits,
                              b.rsum, b.t, b.c)
        assert r.sel[0, 0] == target


# ------------------------------------------------------------------ round

def test_round_is_composition():
    b = synth.config5(G=9, nmin=64, nmax=256)
    o = oracle.round_(b)
    bound, alive = oracle.prune(b.seg_off, b.flops, b.bytes_, b.peak_flops, b.peak_bw, b.incumbent)
    cl = oracle.cluster(b.seg_off, b.koff, b.X, b.iters)
    u = oracle.ucb_select(b.seg_off, b.koff, b.S, cl.assign, alive, bound, b.visits, b.rsum,
                          b.t, b.c)
    np.testing.assert_array_equal(o.alive, alive)
    np.testing.assert_array_equal(o.bound, bound)
    np.testing.assert_array_equal(o.assign, cl.assign)
    np.testing.assert_array_equal(o.cent, cl.cent)
    np.testing.assert_array_equal(o.sel, u.sel)
    np.testing.assert_array_equal(o.ucb, u.ucb)


def test_paper_shape_runs():
    b = synth.paper_shape()
    assert b.N >= 2 * 3          # the |P| >= 2K guard of Alg. 1
    o = oracle.round_(b)
    assert o.counts.sum() == b.N
    assert 0 <= o.sel[0, 0] < 3 and 0 <= o.sel[0, 1] < 6


def test_kstar_tie_goes_to_lowest_candidate():
    r = _ucb_single(2, 1, [1, 0, 1, 1], [1, 1, 1, 1], [3.0, 9.0, 2.0, 2.0],
                    [[1], [5], [1], [1]], [[1], [0], [1], [1]], 8, 1.0)
    np.testing.assert_array_equal(r.sel[0], [1, 0, 2])


def test_prior_is_a_pseudo_count():
    # prior_n pseudo-visits of mean prior_mu: mu = (R + n0*mu0)/(N + n0)
    r = _ucb_single(1, 2, [0], [1], [1.0], [[6, 0]], [[3, 0]], 20, 0.0, pn=2.0, pm=0.75)
    assert abs(r.mu[0, 0] - (3 + 1.5) / 8) < 1e-15
    assert abs(r.mu[0, 1] - 0.75) < 1e-15
    assert abs(r.ucb[0, 1] - 0.75) < 1e-15        # c = 0: no bonus
