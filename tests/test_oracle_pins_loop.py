"""Pins for the oracle's parts that close the loop of Alg. 1 around the scoring
pass: cluster representatives and radii, the strategy mask in the paper's own
form (Eq. 5), masked selection, the draw with the paper's potential, and the
statistics update.  Expected values are hand-worked, closed forms or brute force;
none comes from the oracle or from the GPU path."""
import os

import numpy as np
import pytest
from scipy import stats

import oracle
from paper_2511_18868_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    return [l.split() for l in open(os.path.join(GOLD, name)) if l.strip() and not l.startswith("#")]


def _one(n, k):
    return np.array([0, n], np.int32), np.array([0, k], np.int32)


# ---------------------------------------------------------------- geometry

def test_geometry_hand_example():
    rows = _rows("geometry_hand.txt")
    X = np.array([[float(r[0])] for r in rows], np.float32)
    want_d2 = np.array([float(r[1]) for r in rows])
    seg, koff = _one(len(rows), 1)
    g = oracle.cluster_geometry(seg, koff, X, np.array([[3.2]], np.float32), np.zeros(len(rows), np.int32))
    np.testing.assert_allclose(g.dist2, want_d2, rtol=1e-6)
    assert g.rep[0] == 3
    np.testing.assert_allclose(g.radius[0], 6.8, rtol=1e-6)


def test_geometry_bruteforce_and_covering():
    b = synth.config5(G=7, nmin=64, nmax=400, seed=3)
    c = oracle.cluster(b.seg_off, b.koff, b.X, 4)
    g = oracle.cluster_geometry(b.seg_off, b.koff, b.X, c.cent, c.assign)
    X = b.X.astype(np.float64)
    for s in range(b.G):
        n0, n1, k0, k1 = b.seg_off[s], b.seg_off[s + 1], b.koff[s], b.koff[s + 1]
        for j in range(k1 - k0):
            mem = np.where(c.assign[n0:n1] == j)[0] + n0
            if len(mem) == 0:
                assert g.rep[k0 + j] == -1 and g.radius[k0 + j] == 0.0
                continue
            d = np.sqrt(((X[mem] - c.cent[k0 + j].astype(np.float64)) ** 2).sum(1))
            # the representative is a member and no member is nearer (up to summation order)
            assert g.rep[k0 + j] in mem
            assert d[list(mem).index(g.rep[k0 + j])] <= d.min() * (1 + 1e-12)
            np.testing.assert_allclose(g.radius[k0 + j], d.max(), rtol=1e-12)
            np.testing.assert_allclose(np.sqrt(g.dist2[mem]), d, rtol=1e-12, atol=1e-300)
            # radius <= diameter <= 2 radius (the second by the triangle inequality through
            # the centroid; the first because the centroid is the mean of the members)
            diff = X[mem][:, None, :] - X[mem][None, :, :]
            diam = np.sqrt((diff ** 2).sum(-1)).max()
            assert diam <= 2 * g.radius[k0 + j] * (1 + 1e-12)
            if len(mem) > 1:
                assert diam >= g.radius[k0 + j] * (1 - 1e-6)


def test_geometry_identity_ties_and_empty():
    # every candidate its own cluster: representative = itself, radius 0
    rng = np.random.default_rng(1)
    X = rng.normal(size=(9, 4)).astype(np.float32)
    seg, koff = _one(9, 9)
    g = oracle.cluster_geometry(seg, koff, X, X.copy(), np.arange(9, dtype=np.int32))
    np.testing.assert_array_equal(g.rep, np.arange(9))
    assert (g.radius == 0).all()
    # two members at exactly the same distance: the lower index; an empty cluster: -1
    X = np.array([[5.0, 1.0], [-1.0, 0.0], [1.0, 0.0], [0.0, 3.0]], np.float32)
    seg, koff = _one(4, 3)
    cent = np.array([[0.0, 0.0], [9.0, 9.0], [5.0, 0.0]], np.float32)
    g = oracle.cluster_geometry(seg, koff, X, cent, np.array([2, 0, 0, 0], np.int32))
    np.testing.assert_array_equal(g.rep, [1, -1, 0])
    np.testing.assert_allclose(g.radius, [3.0, 0.0, 1.0])
    # indices are global: a second search starts at its own offset
    seg2 = np.array([0, 4, 8], np.int32)
    koff2 = np.array([0, 3, 6], np.int32)
    g2 = oracle.cluster_geometry(seg2, koff2, np.vstack([X, X]), np.vstack([cent, cent]),
                                 np.array([2, 0, 0, 0, 2, 0, 0, 0], np.int32))
    np.testing.assert_array_equal(g2.rep, [1, -1, 0, 5, -1, 4])


# -------------------------------------------------------------------- mask

def test_strategy_mask_hand_example():
    rows = _rows("strategy_mask_hand.txt")
    h_rep = np.array([[float(v) for v in r[:3]] for r in rows], np.float32)
    want = np.array([[int(v) for v in r[3:]] for r in rows], np.uint8)
    target = np.array([0, 0, 1, 2, 2, 1], np.int32)
    # candidates 0..4; representatives are candidates 3 and 1
    h = np.full((5, 3), 0.99, np.float32)
    h[3] = h_rep[0]
    h[1] = h_rep[1]
    m = oracle.strategy_mask(np.array([0, 2], np.int32), 6, h, target, np.array([3, 1], np.int32), 0.75)
    np.testing.assert_array_equal(m.M, want)
    assert m.nvalid[0] == want.sum()


def test_strategy_mask_extremes_and_counts():
    rng = np.random.default_rng(4)
    koff = np.array([0, 3, 3, 7], np.int32)
    h = rng.uniform(0, 1, (30, 3)).astype(np.float32)
    target = rng.integers(0, 3, 5).astype(np.int32)
    rep = np.array([4, -1, 9, 20, 21, -1, 29], np.int32)
    m = oracle.strategy_mask(koff, 5, h, target, rep, 0.5)
    assert not m.M[rep < 0].any()
    np.testing.assert_array_equal(m.nvalid, [m.M[0:3].sum(), 0, m.M[3:7].sum()])
    brute = np.array([[h[r, target[s]] < np.float32(0.5) if r >= 0 else False for s in range(5)]
                      for r in rep])
    np.testing.assert_array_equal(m.M.astype(bool), brute)
    assert oracle.strategy_mask(koff, 5, h, target, rep, np.inf).M[rep >= 0].all()
    assert not oracle.strategy_mask(koff, 5, h, target, rep, 0.0).M.any()


# ------------------------------------------------------- masked selection

def test_masked_selection():
    b = synth.config5(G=9, nmin=64, nmax=300, S=6, seed=12)
    c = oracle.cluster(b.seg_off, b.koff, b.X, 3)
    bound, alive = oracle.prune(b.seg_off, b.flops, b.bytes_, b.peak_flops, b.peak_bw, b.incumbent)
    base = oracle.ucb_select(b.seg_off, b.koff, b.S, c.assign, alive, bound, b.visits, b.rsum, b.t, b.c)
    ones = np.ones((b.Ksum, b.S), np.uint8)
    same = oracle.ucb_select(b.seg_off, b.koff, b.S, c.assign, alive, bound, b.visits, b.rsum, b.t,
                             b.c, M=ones)
    np.testing.assert_array_equal(same.sel, base.sel)
    np.testing.assert_array_equal(same.ucb, base.ucb)
    # masking the winning arm of every search hands the choice to the runner-up
    M = ones.copy()
    for g in range(b.G):
        I, s = base.sel[g, 0], base.sel[g, 1]
        M[b.koff[g] + I, s] = 0
    r = oracle.ucb_select(b.seg_off, b.koff, b.S, c.assign, alive, bound, b.visits, b.rsum, b.t,
                          b.c, M=M)
    for g in range(b.G):
        tab = base.ucb[b.koff[g]:b.koff[g + 1]].copy()
        tab[M[b.koff[g]:b.koff[g + 1]] == 0] = -np.inf
        flat = int(np.argmax(tab))           # first maximum = lowest flat index
        assert (r.sel[g, 0], r.sel[g, 1]) == (flat // b.S, flat % b.S)
        assert np.isneginf(r.ucb[b.koff[g] + base.sel[g, 0], base.sel[g, 1]])
        k = r.sel[g, 2]
        assert alive[k] and c.assign[k] == r.sel[g, 0]
    # statistics do not depend on the mask
    np.testing.assert_array_equal(r.Ncs, base.Ncs)
    np.testing.assert_array_equal(r.mu, base.mu)
    # nothing valid: no selection
    none = oracle.ucb_select(b.seg_off, b.koff, b.S, c.assign, alive, bound, b.visits, b.rsum, b.t,
                             b.c, M=np.zeros_like(ones))
    assert (none.sel == -1).all()
    # alive = NULL is "all alive"; bound = NULL picks the lowest-index member
    a1 = oracle.ucb_select(b.seg_off, b.koff, b.S, c.assign, None, None, b.visits, b.rsum, b.t, b.c)
    a2 = oracle.ucb_select(b.seg_off, b.koff, b.S, c.assign, np.ones(b.N, np.uint8),
                           np.zeros(b.N, np.float32), b.visits, b.rsum, b.t, b.c)
    np.testing.assert_array_equal(a1.sel, a2.sel)
    np.testing.assert_array_equal(a1.Ncs, a2.Ncs)
    for g in range(b.G):
        mem = np.where(c.assign[b.seg_off[g]:b.seg_off[g + 1]] == a1.sel[g, 0])[0]
        assert a1.sel[g, 2] == b.seg_off[g] + mem[0]


# ------------------------------------------- the draw with the paper's potential

def test_signature_draw_follows_softmax_of_theta_minus_h():
    n, R, theta, tau = 9, 3, 0.75, 0.2
    rng = np.random.default_rng(8)
    h = rng.uniform(0.05, 0.95, (n, R)).astype(np.float32)
    target = np.array([2, 0, 1, 1], np.int32)
    seg = np.array([0, n], np.int32)
    assign = np.zeros(n, np.int32)
    sel = np.array([[0, 1, -1]], np.int32)          # strategy 1 targets resource 0
    V = np.float64(np.float32(theta)) - h[:, 0].astype(np.float64)
    p = np.exp(V / tau)
    p /= p.sum()
    draws = 30000
    cnt = np.zeros(n)
    for d in range(draws):
        cnt[oracle.sample_signature(seg, assign, None, h, target, theta, sel, 5, d, tau).ksel[0]] += 1
    chi2 = ((cnt - draws * p) ** 2 / (draws * p)).sum()
    assert stats.chi2.sf(chi2, n - 1) > 1e-3
    # the other resources' columns play no part; the targeted one does
    for col in (1, 2):
        p_wrong = np.exp((theta - h[:, col].astype(np.float64)) / tau)
        p_wrong /= p_wrong.sum()
        chi2w = ((cnt - draws * p_wrong) ** 2 / (draws * p_wrong)).sum()
        assert stats.chi2.sf(chi2w, n - 1) < 1e-6
    h2 = h.copy()
    h2[:, 1:] = 0.5
    for d in range(50):
        a = oracle.sample_signature(seg, assign, None, h, target, theta, sel, 5, d, tau).ksel
        c = oracle.sample_signature(seg, assign, None, h2, target, theta, sel, 5, d, tau).ksel
        assert a[0] == c[0]
    # same variates as the roofline form: equal potentials give equal draws
    hb = np.repeat((1.0 - h[:, :1]), R, axis=1).astype(np.float32)      # theta - h = V
    for d in range(50):
        a = oracle.sample_signature(seg, assign, None, hb, target, 1.0, sel, 5, d, 1.0).ksel[0]
        c = oracle.sample(seg, assign, None, hb[:, 0], np.array([1.0], np.float32), sel, 5, d, 1.0).ksel[0]
        # V_sig = 1 - hb and V_roof = 1 - hb/1 are the same numbers
        assert a == c


# ------------------------------------------------------------------ update

def test_update_running_mean_closed_form():
    # Alg. 1 starts every arm at N = 1, mu = 0.5 (one pseudo-visit): after rewards
    # r_1..r_T on one arm, mu = (0.5 + sum r) / (1 + T) and N = 1 + T
    S, T = 3, 40
    rng = np.random.default_rng(6)
    rewards = rng.uniform(0, 1, T).astype(np.float32)
    koff = np.array([0, 2], np.int32)
    st = dict(visits=np.zeros((5, S), np.int32), rsum=np.zeros((5, S), np.float32),
              Ncs=np.zeros((2, S), np.int32), mu=np.full((2, S), 0.5, np.float32),
              t=np.array([1], np.int64))
    sel = np.array([[1, 2, -1]], np.int32)
    for i in range(T):
        r = oracle.update_stats(koff, S, sel, np.array([3], np.int32), rewards[i:i + 1],
                                np.array([1], np.uint8), 1.0, **st)
        st = dict(visits=r.visits, rsum=r.rsum, Ncs=r.Ncs, mu=r.mu, t=r.t)
    want = (0.5 + rewards.astype(np.float64).sum()) / (1 + T)
    np.testing.assert_allclose(st["mu"][1, 2], want, rtol=2e-6)
    assert st["Ncs"][1, 2] == T and st["t"][0] == 1 + T
    assert st["visits"][3, 2] == T
    np.testing.assert_allclose(st["rsum"][3, 2], rewards.astype(np.float64).sum(), rtol=2e-6)
    # nothing else moved
    mask = np.ones((2, S), bool); mask[1, 2] = False
    assert (st["mu"][mask] == 0.5).all() and (st["Ncs"][mask] == 0).all()
    st["visits"][3, 2] = 0
    assert not st["visits"].any()


def test_update_skips_unverified_and_unselected():
    S = 2
    koff = np.array([0, 1, 2, 3], np.int32)
    st = dict(visits=np.ones((6, S), np.int32), rsum=np.ones((6, S), np.float32),
              Ncs=np.full((3, S), 4, np.int32), mu=np.full((3, S), 0.25, np.float32),
              t=np.array([7, 8, 9], np.int64))
    sel = np.array([[0, 1, 0], [0, 0, 2], [-1, -1, -1]], np.int32)
    r = oracle.update_stats(koff, S, sel, np.array([1, 2, -1], np.int32),
                            np.array([1.0, 1.0, 1.0], np.float32), np.array([1, 0, 1], np.uint8),
                            0.0, **st)
    np.testing.assert_array_equal(r.t, [8, 9, 10])                       # always
    assert r.Ncs[0, 1] == 5 and r.mu[0, 1] == np.float32(0.25 + 0.75 / 5)
    assert r.visits[1, 1] == 2 and r.rsum[1, 1] == 2.0
    np.testing.assert_array_equal(r.Ncs[1:], st["Ncs"][1:])              # not verified / no arm
    np.testing.assert_array_equal(r.mu[1:], st["mu"][1:])
    np.testing.assert_array_equal(r.visits[2:], st["visits"][2:])


def test_incremental_update_equals_reaggregation():
    # after many updates the incrementally maintained cluster-arm tables equal the
    # tables rebuilt from the per-candidate history (the aggregation of the UCB step)
    b = synth.config5(G=5, nmin=64, nmax=200, S=4, seed=21)
    c = oracle.cluster(b.seg_off, b.koff, b.X, 3)
    agg = oracle.ucb_select(b.seg_off, b.koff, b.S, c.assign, None, None, b.visits, b.rsum, b.t, b.c)
    st = dict(visits=b.visits, rsum=b.rsum, Ncs=agg.Ncs.astype(np.int32),
              mu=agg.mu.astype(np.float32), t=b.t)
    rng = np.random.default_rng(0)
    for it in range(60):
        sel = np.zeros((b.G, 3), np.int32)
        ksel = np.zeros(b.G, np.int32)
        for g in range(b.G):
            k = rng.integers(b.seg_off[g], b.seg_off[g + 1])
            sel[g] = (c.assign[k], rng.integers(0, b.S), -1)
            ksel[g] = k
        r = oracle.update_stats(b.koff, b.S, sel, ksel, rng.uniform(0, 1, b.G).astype(np.float32),
                                (rng.random(b.G) < 0.8).astype(np.uint8), 0.0, **st)
        st = dict(visits=r.visits, rsum=r.rsum, Ncs=r.Ncs, mu=r.mu, t=r.t)
    agg2 = oracle.ucb_select(b.seg_off, b.koff, b.S, c.assign, None, None, st["visits"], st["rsum"],
                             st["t"], b.c)
    np.testing.assert_array_equal(st["Ncs"], agg2.Ncs)
    np.testing.assert_allclose(st["mu"], agg2.mu, rtol=2e-5)
    np.testing.assert_array_equal(st["t"], b.t + 60)


# ----------------------------------------------------------------- seeding

def test_seed_farthest_hand_example():
    rows = _rows("seed_farthest_hand.txt")
    X = np.array([[float(r[0])] for r in rows], np.float32)
    order = [int(r[1]) for r in rows]
    K = max(order) + 1
    want_pick = [order.index(j) for j in range(K)]
    seg, koff = _one(len(rows), K)
    s = oracle.seed_farthest(seg, koff, X)
    np.testing.assert_array_equal(s.pick, want_pick)
    np.testing.assert_array_equal(s.cent[:, 0], X[want_pick, 0])


def test_seed_farthest_greedy_property_and_two_approximation():
    # every pick maximises the distance to the picks before it (checked with numpy),
    # and the greedy cover's radius is within a factor two of the best possible
    # k-centre radius over all K-subsets of the rows (brute force)
    import itertools
    rng = np.random.default_rng(3)
    for trial in range(6):
        n, D, K = 11, 3, 3
        X = rng.normal(size=(n, D)).astype(np.float32)
        seg, koff = _one(n, K)
        s = oracle.seed_farthest(seg, koff, X)
        X64 = X.astype(np.float64)
        d2 = ((X64[:, None, :] - X64[None, :, :]) ** 2).sum(-1)
        assert s.pick[0] == 0
        for j in range(1, K):
            mind = d2[:, s.pick[:j]].min(1)
            assert mind[s.pick[j]] >= mind.max() * (1 - 1e-12)
        np.testing.assert_array_equal(s.cent, X[s.pick])
        greedy_r = np.sqrt(d2[:, s.pick].min(1).max())
        best_r = min(np.sqrt(d2[:, list(c)].min(1).max()) for c in itertools.combinations(range(n), K))
        assert greedy_r <= 2 * best_r * (1 + 1e-9)


def test_seed_farthest_segments_duplicates_and_radius_gain():
    # global indices per search; with fewer distinct rows than clusters the first row
    # is taken again once the farthest distance is zero
    X = np.array([[0.0], [0.0], [5.0], [7.0], [7.0], [9.0]], np.float32)
    seg = np.array([0, 3, 6], np.int32)
    koff = np.array([0, 3, 5], np.int32)
    s = oracle.seed_farthest(seg, koff, X)
    np.testing.assert_array_equal(s.pick, [0, 2, 0, 3, 5])
    # scaling by a power of two scales every distance exactly: same picks at any scale
    for e in (-12, 9):
        np.testing.assert_array_equal(oracle.seed_farthest(seg, koff, X * np.float32(2.0 ** e)).pick, s.pick)
    # on blobs the greedy cover starts Lloyd from a smaller covering radius than the
    # first K rows do
    b = synth.config5(G=6, nmin=200, nmax=600, seed=40)
    far = oracle.seed_farthest(b.seg_off, b.koff, b.X)
    first = np.vstack([b.X[b.seg_off[g]:b.seg_off[g] + (b.koff[g + 1] - b.koff[g])] for g in range(b.G)])
    def cover(cent):
        a, mind2, _ = oracle.assign(b.seg_off, b.koff, b.X, cent)
        return np.array([np.sqrt(mind2[b.seg_off[g]:b.seg_off[g + 1]].max()) for g in range(b.G)])
    assert (cover(far.cent) < cover(first)).all()


def test_seed_dsquared_first_two_draws_follow_their_laws():
    # first centroid: uniform over the rows; second: P(k) = D_k^2 / sum D^2 given the first
    n, D = 9, 2
    rng = np.random.default_rng(12)
    X = rng.normal(size=(n, D)).astype(np.float32)
    seg, koff = _one(n, 2)
    draws = 24000
    first = np.zeros(n)
    second = np.zeros((n, n))
    for d in range(draws):
        s = oracle.seed_dsquared(seg, koff, X, 2024, 1000 * d)
        first[s.pick[0]] += 1
        second[s.pick[0], s.pick[1]] += 1
        assert s.pick[0] != s.pick[1]                      # a chosen row has weight zero
    chi2 = ((first - draws / n) ** 2 / (draws / n)).sum()
    assert stats.chi2.sf(chi2, n - 1) > 1e-3
    X64 = X.astype(np.float64)
    d2 = ((X64[:, None, :] - X64[None, :, :]) ** 2).sum(-1)
    for a in range(n):
        p = d2[a] / d2[a].sum()
        m = first[a]
        keep = p > 0
        chi2 = ((second[a][keep] - m * p[keep]) ** 2 / (m * p[keep])).sum()
        assert stats.chi2.sf(chi2, keep.sum() - 1) > 1e-4, (a, chi2)
        # a uniform second draw would be rejected
        chi2u = ((second[a][keep] - m / (n - 1)) ** 2 / (m / (n - 1))).sum()
        assert stats.chi2.sf(chi2u, keep.sum() - 1) < 1e-6


def test_seed_dsquared_structure():
    b = synth.config5(G=5, nmin=64, nmax=300, seed=9)
    s = oracle.seed_dsquared(b.seg_off, b.koff, b.X, 7, 3)
    for g in range(b.G):
        pk = s.pick[b.koff[g]:b.koff[g + 1]]
        assert ((pk >= b.seg_off[g]) & (pk < b.seg_off[g + 1])).all()
        assert len(set(pk.tolist())) == len(pk)            # distinct rows: no duplicates in this data
    np.testing.assert_array_equal(s.cent, b.X[s.pick])
    # reproducible; another seed or draw number gives other seeds
    s2 = oracle.seed_dsquared(b.seg_off, b.koff, b.X, 7, 3)
    np.testing.assert_array_equal(s.pick, s2.pick)
    assert (oracle.seed_dsquared(b.seg_off, b.koff, b.X, 8, 3).pick != s.pick).any()
    assert (oracle.seed_dsquared(b.seg_off, b.koff, b.X, 7, 4).pick != s.pick).any()
    # identical rows: after the first pick every weight is zero and the draw falls back to
    # the lowest index
    X = np.ones((6, 3), np.float32)
    seg, koff = _one(6, 3)
    d = oracle.seed_dsquared(seg, koff, X, 1, 0)
    assert d.pick[1] == 0 and d.pick[2] == 0
    # mean D^2 cost of the seeds is below that of the first K rows on blobs (the point of ++)
    far = []
    for draw in range(5):
        sd = oracle.seed_dsquared(b.seg_off, b.koff, b.X, 5, 100 * draw)
        _, m2, _ = oracle.assign(b.seg_off, b.koff, b.X, sd.cent)
        far.append(m2.sum())
    first = np.vstack([b.X[b.seg_off[g]:b.seg_off[g] + (b.koff[g + 1] - b.koff[g])] for g in range(b.G)])
    _, m1, _ = oracle.assign(b.seg_off, b.koff, b.X, first)
    assert np.mean(far) < m1.sum()


# --------------------------------------------------------------- diameters

def test_diameter_hand_example():
    rows = _rows("diameter_hand.txt")
    X = np.array([[float(r[0]), float(r[1])] for r in rows], np.float32)
    a = np.array([int(r[2]) for r in rows], np.int32)
    seg, koff = _one(len(rows), 4)            # cluster 3 has no member
    np.testing.assert_allclose(oracle.cluster_diameter(seg, koff, X, a), [5.0, 0.0, 7.0, 0.0])


def test_diameter_bruteforce_radius_relation_and_invariance():
    b = synth.config5(G=6, nmin=64, nmax=400, seed=33)
    c = oracle.cluster(b.seg_off, b.koff, b.X, 4)
    diam = oracle.cluster_diameter(b.seg_off, b.koff, b.X, c.assign)
    X = b.X.astype(np.float64)
    for s in range(b.G):
        n0, n1, k0 = b.seg_off[s], b.seg_off[s + 1], b.koff[s]
        for j in range(b.koff[s + 1] - k0):
            mem = np.where(c.assign[n0:n1] == j)[0] + n0
            if len(mem) < 2:
                assert diam[k0 + j] == 0.0
                continue
            diff = X[mem][:, None, :] - X[mem][None, :, :]
            np.testing.assert_allclose(diam[k0 + j], np.sqrt((diff ** 2).sum(-1)).max(), rtol=1e-12)
    # against the independent radius computation: radius <= diam <= 2 radius, with the
    # centroids that are the means of these members
    upd, _ = oracle.update(b.seg_off, b.koff, b.X, c.cent, c.assign)
    geo = oracle.cluster_geometry(b.seg_off, b.koff, b.X, upd, c.assign)
    many = c.counts > 1
    assert (diam[many] <= 2 * geo.radius[many] * (1 + 1e-6)).all()
    assert (diam[many] >= geo.radius[many] * (1 - 1e-6)).all()
    # a shift of all rows by a constant vector leaves every diameter unchanged
    # (integers keep the shift exact in fp32)
    Xi = np.round(b.X * 64).astype(np.float32)
    d1 = oracle.cluster_diameter(b.seg_off, b.koff, Xi, c.assign)
    d2 = oracle.cluster_diameter(b.seg_off, b.koff, Xi + np.float32(1000.0), c.assign)
    np.testing.assert_array_equal(d1, d2)
    # members of other searches or clusters play no part
    a2 = c.assign.copy()
    np.testing.assert_array_equal(oracle.cluster_diameter(b.seg_off, b.koff, b.X, a2), diam)
    seg1 = np.array([0, b.seg_off[1]], np.int32)
    koff1 = np.array([0, b.koff[1]], np.int32)
    np.testing.assert_array_equal(
        oracle.cluster_diameter(seg1, koff1, b.X[:b.seg_off[1]], c.assign[:b.seg_off[1]]),
        diam[:b.koff[1]])
