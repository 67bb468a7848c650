"""Pins of the oracle's near-tie flags ("any near-tie within 1e-6 flagged and
excluded").  The flags decide which candidates and searches the GPU parity
tests leave out of the bit-exact comparisons, so the threshold itself has to be
fixed: every case here places a runner-up at a hand-chosen relative gap just
below and just above 1e-6 of the reference value, and once at another scale, so
that a threshold outside (0.9e-6, 1.1e-6) - or an absolute instead of a relative
one - fails."""
import math

import numpy as np
import pytest

import oracle


def _one(n, k):
    return np.array([0, n], np.int32), np.array([0, k], np.int32)


# ----------------------------------------------------- nearest-centroid flag

def _gap_case(scale, rel):
    """A candidate x = (scale, 0) between c0 = (0, 0) and c1 = (0, b): squared
    distances scale^2 and scale^2 + b^2, so the relative gap of the runner-up is
    b^2 / (scale^2 + b^2).  Returns fp32 inputs and the gap they really have."""
    b = np.float32(scale * math.sqrt(rel / (1.0 - rel)))
    x = np.array([[scale, 0.0]], np.float32)
    cin = np.array([[0.0, 0.0], [0.0, b]], np.float32)
    d0 = float(x[0, 0]) ** 2
    d1 = d0 + float(b) ** 2
    return x, cin, (d1 - d0) / d1


@pytest.mark.parametrize("scale", [1.0, 1000.0, 1.0 / 1024])
def test_assign_flag_threshold_is_1e6_relative(scale):
    seg, ko = _one(1, 2)
    for rel, want in ((0.5e-6, 1), (0.95e-6, 1), (1.05e-6, 0), (5e-6, 0), (1e-3, 0)):
        x, cin, real = _gap_case(scale, rel)
        assert abs(real / rel - 1) < 1e-3                 # the inputs have the intended gap
        r = oracle.cluster_step(seg, ko, x, cin)
        assert r.assign[0] == 0
        assert r.flag[0] == want, (scale, rel)


def test_assign_flag_between_fp32_neighbours():
    # 1-D, centroids 0 and 2: x = 1 + m ulp has squared distances (1 +- m 2^-23)^2, a
    # relative gap of about 4 m 2^-23 = m * 4.77e-7: m = 1, 2 flag, m = 3 does not
    seg, ko = _one(4, 2)
    cin = np.array([[0.0], [2.0]], np.float32)
    x = (1.0 + np.array([[0], [1], [2], [3]]) * 2.0 ** -23).astype(np.float32)
    r = oracle.cluster_step(seg, ko, x, cin)
    np.testing.assert_array_equal(r.flag, [1, 1, 1, 0])
    np.testing.assert_array_equal(r.assign, [0, 1, 1, 1])


# ------------------------------------------------------------ selection flag

def _two_arms(n0, r0, n1, r1, **kw):
    """One search, two clusters of one candidate each, one strategy, t = 1 (no
    exploration bonus): the scores are the mean rewards r/n."""
    seg, ko = _one(2, 2)
    return oracle.ucb_select(seg, ko, 1, np.array([0, 1], np.int32), np.ones(2, np.uint8),
                             np.array([1.0, 2.0], np.float32),
                             np.array([[n0], [n1]], np.int32), np.array([[r0], [r1]], np.float32),
                             np.array([1], np.int64), 2.0, **kw)


def test_selection_flag_threshold_is_1e6_relative_to_the_best_score():
    n = 10_000_000                                   # below 2^24: the reward sums are exact in fp32
    # best score 1.0, runner-up 1 - m 1e-7
    for m, want in ((0, 0), (5, 1), (9, 1), (11, 0), (50, 0), (10_000, 0)):
        r = _two_arms(n, n, n, n - m)
        assert r.near[0] == want, m
        np.testing.assert_array_equal(r.sel[0][:2], [0, 0])
    # best score 0.5: a gap of 6e-7 is 1.2e-6 of it (not flagged; an absolute threshold
    # would flag), a gap of 4e-7 is 0.8e-6 (flagged)
    assert _two_arms(n, n // 2, n, n // 2 - 6).near[0] == 0
    assert _two_arms(n, n // 2, n, n // 2 - 4).near[0] == 1
    # the better arm second: same flags, the other cluster selected
    r = _two_arms(n, n - 9, n, n)
    assert r.near[0] == 1 and tuple(r.sel[0][:2]) == (1, 0)
    assert _two_arms(n, n - 11, n, n).near[0] == 0


# --------------------------------------------------- flags of the two draws

def _gumbel(seed, draw, k):
    u = oracle.uniform(seed, draw, k)
    return -math.log(-math.log(u))


def test_draw_flag_threshold_is_1e6_relative_to_the_best_key():
    # Two alive members in the chosen cluster.  Keys V/tau + g with the variates g of
    # (seed, draw); tau = 64 makes the fp32 headroom fine enough to place the second
    # key at a chosen distance below the first.
    # (a draw whose two variates are close is looked for, so that the headroom that
    # makes up their difference is small and its fp32 rounding is far below the gap)
    seed, tau = 77, 64.0
    seg = np.array([0, 2], np.int32)
    a = np.zeros(2, np.int32)
    sel = np.array([[0, 0, 0]], np.int32)
    inc = np.array([1.0], np.float32)
    draw = next(d for d in range(100000)
                if abs(_gumbel(seed, d, 0) - _gumbel(seed, d, 1)) < 2e-3 and abs(_gumbel(seed, d, 0)) > 0.5)
    g0, g1 = _gumbel(seed, draw, 0), _gumbel(seed, draw, 1)
    for rel, want in ((0.5e-6, 1), (0.9e-6, 1), (1.1e-6, 0), (1e-4, 0)):
        # candidate 0: bound 0.5 -> V = 0.5; candidate 1: V1 so that key1 = key0 - rel |key0|
        key0 = 0.5 / tau + g0
        v1 = (key0 - rel * abs(key0) - g1) * tau
        bound = np.array([0.5, 1.0 - v1], np.float32)
        # what the fp32 inputs really give
        k0 = (1.0 - float(bound[0]) / 1.0) / tau + g0
        k1 = (1.0 - float(bound[1]) / 1.0) / tau + g1
        real = (k0 - k1) / abs(k0)
        assert abs(real / rel - 1) < 0.03, (real, rel)
        r = oracle.sample(seg, a, None, bound, inc, sel, seed, draw, tau)
        assert r.ksel[0] == 0 and r.near[0] == want, rel


def test_dsquared_seeding_flag_threshold():
    # Three rows in two features.  Whichever row the first (uniform) draw takes, the two
    # others compete in the second draw with keys ln D^2 + g.  One of them sits at
    # distance 1; the other is placed so that its key lies a chosen relative distance
    # below: D^2 = p^2 + q^2 with q the fine adjustment (fp32 coordinates).
    seed, draw0 = 2511, 40
    seg, ko = _one(3, 2)
    first = int(np.argmax([_gumbel(seed, draw0, k) for k in range(3)]))
    ra, rb = [k for k in range(3) if k != first]
    ga, gb = _gumbel(seed, draw0 + 1, ra), _gumbel(seed, draw0 + 1, rb)
    for rel, want in ((0.5e-6, 1), (0.9e-6, 1), (1.1e-6, 0), (1e-4, 0)):
        key_a = 0.0 + ga                                  # ln 1 + g
        target = math.exp(key_a - rel * abs(key_a) - gb)  # D^2 of row rb
        p = np.nextafter(np.float32(math.sqrt(target)), np.float32(0))
        q = np.float32(math.sqrt(max(target - float(p) ** 2, 0.0)))
        X = np.zeros((3, 2), np.float32)
        X[ra] = [1.0, 0.0]
        X[rb] = [0.0, 0.0]
        X[rb, 0], X[rb, 1] = -p, q
        d2b = float(p) ** 2 + float(q) ** 2
        real = (key_a - (math.log(d2b) + gb)) / abs(key_a)
        assert abs(real / rel - 1) < 0.03, (real, rel)
        r = oracle.seed_dsquared(seg, ko, X, seed, draw0)
        np.testing.assert_array_equal(r.pick, [first, ra])
        assert r.near[0] == want, rel
