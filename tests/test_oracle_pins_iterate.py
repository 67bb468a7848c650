"""Pins of the oracle's composition of whole iterations of Alg. 1
(oracle.iterate): bookkeeping that must hold whatever the arithmetic of the
stages (each pinned in its own file) - the iteration counter, what the update
adds where, when re-clustering happens and which searches it leaves alone."""
import numpy as np

import oracle
from paper_2511_18868_amd import synth


def _setup(b, rounds, seed=0):
    h, target, theta = synth.signatures(b, 3)
    rw, ok = zip(*[synth.feedback(b, seed=seed * 1000 + r) for r in range(rounds)])
    return h, target, theta, np.stack(rw), np.stack(ok)


def _run(b, rounds, tau, t0, warm, state=None, iters=3, seed=0):
    h, target, theta, rw, ok = _setup(b, rounds, seed)
    if state is None:
        cl = oracle.cluster(b.seg_off, b.koff, b.X, 2)
        geo = oracle.cluster_geometry(b.seg_off, b.koff, b.X, cl.cent, cl.assign)
        M = oracle.strategy_mask(b.koff, b.S, h, target, geo.rep, theta).M
        state = (cl.assign, cl.cent, cl.counts, cl.objective, geo.rep, M)
    out = oracle.iterate(b.seg_off, b.koff, b.S, b.X, h, target, theta, None, rw, ok, b.visits,
                         b.rsum, b.t, *state, rounds, tau, t0, warm, iters, b.c, 1.0, 0.5,
                         seed=99, draw0=7)
    return out, (h, target, theta, rw, ok), state


def test_counters_and_history_advance_as_alg1_states():
    b = synth.config5(G=12, nmin=64, nmax=200, S=6, seed=41)
    T = 9
    out, (h, target, theta, rw, ok), _ = _run(b, T, 0, 0, 0)
    np.testing.assert_array_equal(out.t, b.t + T)                      # t advances every iteration
    dv = out.visits.astype(np.int64) - b.visits
    dr = out.rsum.astype(np.float64) - b.rsum
    assert (dv >= 0).all()
    sid = np.repeat(np.arange(b.G), np.diff(b.seg_off))
    for g in range(b.G):
        chosen = out.sel_log[:, g, 0] >= 0
        good = chosen & (ok[:, g] != 0) & (out.ksel_log[:, g] >= 0)
        assert dv[sid == g].sum() == good.sum()                        # one visit per verified kernel
        assert abs(dr[sid == g].sum() - rw[good, g].astype(np.float64).sum()) < 1e-4
        for r in np.where(good)[0]:
            k, s = out.ksel_log[r, g], out.sel_log[r, g, 1]
            assert b.seg_off[g] <= k < b.seg_off[g + 1]                # the drawn kernel is in the search ...
            assert dv[k, s] >= 1                                       # ... and its arm was visited
            assert out.assign[k] == out.sel_log[r, g, 0]               # ... in the chosen cluster
    # nothing was re-clustered
    cl = oracle.cluster(b.seg_off, b.koff, b.X, 2)
    np.testing.assert_array_equal(out.assign, cl.assign)


def test_first_round_equals_the_stages_called_one_by_one():
    b = synth.config5(G=7, nmin=64, nmax=150, S=5, seed=42)
    out, (h, target, theta, rw, ok), st = _run(b, 1, 0, 0, 0)
    u = oracle.ucb_select(b.seg_off, b.koff, b.S, st[0], None, None, b.visits, b.rsum, b.t, b.c, 1.0,
                          0.5, M=st[5])
    s = oracle.sample_signature(b.seg_off, st[0], None, h, target, theta, u.sel, 99, 7, 1.0)
    np.testing.assert_array_equal(out.sel_log[0], u.sel)
    np.testing.assert_array_equal(out.ksel_log[0], s.ksel)
    up = oracle.update_stats(b.koff, b.S, u.sel, s.ksel, rw[0], ok[0], 1.0, b.visits, b.rsum,
                             u.Ncs.astype(np.int32), u.mu.astype(np.float32), b.t)
    np.testing.assert_array_equal(out.visits, up.visits)
    np.testing.assert_array_equal(out.mu, up.mu)


def test_reclustering_happens_when_the_iteration_number_is_a_multiple_of_tau():
    b = synth.config5(G=6, nmin=100, nmax=200, S=4, seed=43)
    h, target, theta, rw, ok = _setup(b, 12)
    # a stale state: everything in cluster 0, so only cluster 0 has members
    stale = (np.zeros(b.N, np.int32), np.zeros((b.Ksum, b.D), np.float32),
             np.zeros(b.Ksum, np.int32), np.zeros(b.G), np.full(b.Ksum, -1, np.int32),
             np.ones((b.Ksum, b.S), np.uint8))
    for g in range(b.G):
        stale[4][b.koff[g]] = b.seg_off[g]
    out = oracle.iterate(b.seg_off, b.koff, b.S, b.X, h, target, theta, None, rw, ok, b.visits,
                         b.rsum, b.t, *stale, 12, 10, 3, 0, 3, b.c, 1.0, 0.5, seed=5, draw0=0)
    # iterations 3..9 run on the stale state (only cluster 0 can be chosen); iteration
    # 10 = round 7 re-clusters, after which other clusters are chosen too
    assert (out.sel_log[:7, :, 0] == 0).all()
    assert (out.sel_log[7:, :, 0] > 0).any()
    want = oracle.cluster(b.seg_off, b.koff, b.X, 3)
    np.testing.assert_array_equal(out.assign, want.assign)
    np.testing.assert_array_equal(out.counts, want.counts)


def test_searches_with_fewer_than_2k_candidates_keep_their_clustering():
    b = synth.config5(G=5, nmin=64, nmax=120, S=4, seed=44)
    # raise K of search 1 above N/2: koff rebuilt
    kg = np.diff(b.koff).copy()
    ng = np.diff(b.seg_off)
    kg[1] = ng[1] // 2 + 1
    b.koff = np.concatenate([[0], np.cumsum(kg)]).astype(np.int32)
    out, _, st = _run(b, 2, 1, 0, 1, iters=2)     # re-cluster in both rounds, warm start
    sl = slice(b.seg_off[1], b.seg_off[2])
    kl = slice(b.koff[1], b.koff[2])
    np.testing.assert_array_equal(out.assign[sl], st[0][sl])
    np.testing.assert_array_equal(out.cent[kl], st[1][kl])
    np.testing.assert_array_equal(out.counts[kl], st[2][kl])
    # the others went through 2 + 2 + 2 Lloyd steps in all (warm start continues)
    want = oracle.cluster(b.seg_off, b.koff, b.X, 6)
    for g in (0, 2, 3, 4):
        s2 = slice(b.seg_off[g], b.seg_off[g + 1])
        if not want.dirty[g]:
            np.testing.assert_array_equal(out.assign[s2], want.assign[s2])
