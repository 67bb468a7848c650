"""Pins for the oracle's draw of k_t inside the chosen cluster (Sec. 3.4, Alg. 1
"Sample k_t"): the published known answers of the counter-based generator, the
distribution the Gumbel-max identity must reproduce (softmax over the headroom),
its limits in the temperature, and membership invariants.  None of the expected
values comes from the oracle or from the GPU path."""
import os

import numpy as np
import pytest
from scipy import stats

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _kat_rows():
    rows = []
    for line in open(os.path.join(GOLD, "philox4x32_10_kat.txt")):
        if line.strip() and not line.startswith("#"):
            w = [int(x, 16) for x in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert oracle.philox4x32_10(ctr, key) == want


def test_uniform_uses_the_documented_words():
    # counter (k, 0, draw lo, draw hi), key (seed lo, seed hi): the all-zero known
    # answer fixes the variate of candidate 0 in draw 0 under seed 0 ...
    _, _, out = _kat_rows()[0]
    m = (out[0] << 20) | (out[1] >> 12)
    assert oracle.uniform(0, 0, 0) == (m + 0.5) / 2.0 ** 52
    # ... and the pi vector fixes where k, draw and seed go
    want = oracle.philox4x32_10([7, 0, 0x89abcdef, 0x01234567], [0x55aa55aa, 0x0badcafe])
    m = (want[0] << 20) | (want[1] >> 12)
    assert oracle.uniform(0x0badcafe55aa55aa, 0x0123456789abcdef, 7) == (m + 0.5) / 2.0 ** 52


def test_uniform_is_uniform_and_independent():
    u_k = np.array([oracle.uniform(11, 3, k) for k in range(20000)])
    u_d = np.array([oracle.uniform(11, d, 5) for d in range(20000)])
    u_s = np.array([oracle.uniform(s, 3, 5) for s in range(20000)])
    for u in (u_k, u_d, u_s):
        assert u.min() > 0.0 and u.max() < 1.0
        assert stats.kstest(u, "uniform").pvalue > 1e-3
        assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.03
    assert abs(np.corrcoef(u_k, u_d)[0, 1]) < 0.03


def _one_cluster(n, bound, inc, alive=None):
    seg = np.array([0, n], np.int32)
    assign = np.zeros(n, np.int32)
    sel = np.array([[0, 0, -1]], np.int32)
    return seg, assign, alive, np.asarray(bound, np.float32), np.array([inc], np.float32), sel


def _freq(args, n, tau, draws, seed=20251118):
    cnt = np.zeros(n)
    for d in range(draws):
        cnt[oracle.sample(*args, seed, d, tau).ksel[0]] += 1
    return cnt


@pytest.mark.parametrize("tau", [1.0, 0.25])
def test_sampling_frequencies_follow_the_softmax_of_the_headroom(tau):
    # P(k) = exp(V_k/tau) / sum exp(V/tau), V_k = 1 - bound_k / incumbent
    n, inc = 10, 2.0
    bound = np.linspace(0.1, 1.9, n)
    args = _one_cluster(n, bound, inc)
    V = 1.0 - np.float32(bound).astype(np.float64) / inc
    p = np.exp(V / tau)
    p /= p.sum()
    draws = 30000
    cnt = _freq(args, n, tau, draws)
    assert cnt.sum() == draws
    chi2 = ((cnt - draws * p) ** 2 / (draws * p)).sum()
    assert stats.chi2.sf(chi2, n - 1) > 1e-3, (chi2, cnt, draws * p)
    # the tilt is in the right direction and of the right size: most headroom first
    assert cnt[0] > cnt[-1]
    # a uniform law, the reversed tilt and a tilt without the temperature are all rejected
    for wrong in (np.full(n, 1.0 / n), p[::-1], np.exp(V) / np.exp(V).sum()):
        if np.allclose(wrong, p):
            continue
        chi2w = ((cnt - draws * wrong) ** 2 / (draws * wrong)).sum()
        assert stats.chi2.sf(chi2w, n - 1) < 1e-6


def test_zero_temperature_limit_is_the_largest_headroom():
    rng = np.random.default_rng(5)
    n = 50
    bound = rng.uniform(0.1, 0.9, n)
    args = _one_cluster(n, bound, 1.0)
    for d in range(20):
        assert oracle.sample(*args, 1, d, 1e-9).ksel[0] == int(np.argmin(np.float32(bound)))
    # at a temperature so low that the variates are absorbed, equal headrooms tie
    # exactly: the lowest index wins
    bound[[7, 31, 44]] = 0.05
    args = _one_cluster(n, bound, 1.0)
    for d in range(20):
        assert oracle.sample(*args, 1, d, 1e-300).ksel[0] == 7


def test_infinite_incumbent_and_high_temperature_are_uniform():
    n = 8
    bound = np.geomspace(1e-3, 1.0, n)
    for args, tau in ((_one_cluster(n, bound, np.inf), 1.0), (_one_cluster(n, bound, 2.0), 1e9)):
        draws = 16000
        cnt = _freq(args, n, tau, draws)
        chi2 = ((cnt - draws / n) ** 2 / (draws / n)).sum()
        assert stats.chi2.sf(chi2, n - 1) > 1e-3


def test_sample_is_an_alive_member_of_the_chosen_cluster():
    rng = np.random.default_rng(9)
    G, S = 6, 3
    sizes = np.array([40, 0, 17, 64, 5, 33])
    seg = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    N = int(seg[-1])
    K = np.array([4, 1, 2, 5, 1, 3])
    assign = np.concatenate([rng.integers(0, k, n) for k, n in zip(K, sizes)]).astype(np.int32)
    alive = (rng.random(N) < 0.6).astype(np.uint8)
    bound = rng.uniform(0.1, 0.9, N).astype(np.float32)
    inc = np.ones(G, np.float32)
    sel = np.array([[1, 0, -1], [-1, -1, -1], [0, 2, -1], [4, 1, -1], [0, 0, -1], [2, 2, -1]], np.int32)
    # search 4: make sure nothing is alive in the chosen cluster
    alive[seg[4]:seg[5]] = 0
    seen = [set() for _ in range(G)]
    for d in range(200):
        r = oracle.sample(seg, assign, alive, bound, inc, sel, 77, d, 1.0)
        for g in range(G):
            k = r.ksel[g]
            members = [q for q in range(seg[g], seg[g + 1]) if alive[q] and assign[q] == sel[g, 0]]
            if sel[g, 0] < 0 or not members:
                assert k == -1
            else:
                assert k in members
                seen[g].add(int(k))
    # different draws visit different members; the same (seed, draw) repeats itself
    assert len(seen[0]) > 1 and len(seen[3]) > 1
    a = oracle.sample(seg, assign, alive, bound, inc, sel, 77, 5, 1.0).ksel
    b = oracle.sample(seg, assign, alive, bound, inc, sel, 77, 5, 1.0).ksel
    np.testing.assert_array_equal(a, b)
    # candidates outside the chosen cluster have no influence
    bound2 = bound.copy()
    out = np.ones(N, bool)
    for g in range(G):
        out[seg[g]:seg[g + 1]] = assign[seg[g]:seg[g + 1]] != sel[g, 0]
    bound2[out] *= 0.5
    c = oracle.sample(seg, assign, alive, bound2, inc, sel, 77, 5, 1.0).ksel
    np.testing.assert_array_equal(a, c)
    # alive = NULL means every candidate is alive
    d_all = oracle.sample(seg, assign, None, bound, inc, sel, 77, 5, 1.0).ksel
    d_one = oracle.sample(seg, assign, np.ones(N, np.uint8), bound, inc, sel, 77, 5, 1.0).ksel
    np.testing.assert_array_equal(d_all, d_one)
    assert d_all[4] >= 0


def test_single_member_is_always_drawn():
    seg, assign, _, bound, inc, sel = _one_cluster(9, np.linspace(0.1, 0.9, 9), 1.0)
    alive = np.zeros(9, np.uint8)
    alive[6] = 1
    for d in range(10):
        r = oracle.sample(seg, assign, alive, bound, inc, sel, 3, d, 1.0)
        assert r.ksel[0] == 6 and r.near[0] == 0


def test_near_flag_matches_keys_recomputed_independently():
    # the keys V/tau - ln(-ln u) recomputed with numpy from the generator's variates:
    # the flag is set exactly when the two largest are within 1e-6 relative
    n, inc, tau = 400, 1.0, 0.5
    rng = np.random.default_rng(2)
    bound = rng.uniform(0.1, 0.9, n).astype(np.float32)
    args = _one_cluster(n, bound, inc)
    flagged = 0
    for d in range(300):
        r = oracle.sample(*args, 99, d, tau)
        u = np.array([oracle.uniform(99, d, k) for k in range(n)])
        key = (1.0 - bound.astype(np.float64) / inc) / tau - np.log(-np.log(u))
        o = np.argsort(-key, kind="stable")
        gap = key[o[0]] - key[o[1]]
        if gap > 1e-5 * abs(key[o[0]]):
            assert r.ksel[0] == o[0] and r.near[0] == 0
        elif gap < 1e-7 * abs(key[o[0]]):
            assert r.near[0] == 1
        flagged += int(r.near[0])
    assert flagged <= 2
