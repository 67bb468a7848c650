"""A sweep over feature counts, cluster counts and search lengths around the
kernels' internal boundaries (16-feature steps of the matrix instruction,
centroid tiles of 32, candidate tiles of 32, the 16-byte row pieces), each shape
through a whole kb_round and compared with the oracle: masks, assignments and
selections bit for bit on the searches the oracle saw no near-tie in, centroids
and scores within the stated tolerance."""
import numpy as np
import pytest

import oracle
from paper_2511_18868_amd import synth
from kbcheck import assert_cent_close, assert_rel_close, search_of

pytestmark = pytest.mark.gpu

# cluster counts around the centroid-tile boundaries of the one-workgroup kernel
KS = (1, 2, 5, 16, 31, 32, 33, 48, 63, 64)


@pytest.fixture(scope="module")
def kb():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2511_18868_amd import binding
    binding.lib()
    return binding


def _batch(D, S, seed, many=False):
    """One search per cluster count, lengths with ragged tails (not multiples of 32).
    many: followed by 250 short searches, so that the batch holds more searches than
    the chip has compute units and the one-workgroup kernel runs its 256-thread shape."""
    rng = np.random.default_rng(seed)
    b = None
    for i, K in enumerate(KS):
        n = int(rng.integers(3 * K + 1, 40 * K + 40))
        one = synth.config2(seed=seed * 100 + i, N=n, D=D, K=K, S=S, iters=6)
        b = one if b is None else synth.concat(b, one, f"sweepD{D}")
    if many:
        b = synth.concat(b, synth.config5(G=250, nmin=17, nmax=90, D=D, S=S, iters=6, seed=seed + 7),
                         f"sweepD{D}many")
    return b


# feature counts: one to four 16-feature steps, with and without padding; 6 and 17
# are not multiples of 4: rows are then fetched feature by feature
@pytest.mark.parametrize("D", [4, 6, 8, 12, 16, 17, 20, 28, 32, 36, 44, 48, 52, 60, 64])
@pytest.mark.parametrize("scorer", [0, 2], ids=["bounds", "matrixcore"])
@pytest.mark.parametrize("many", [False, True], ids=["few", "many"])
def test_round_over_shapes(kb, D, scorer, many):
    import torch
    S = 3 if D % 8 == 4 else 4            # (an odd strategy count takes the scalar row path of the selection)
    b = _batch(D, S, seed=1000 + D, many=many)
    d = kb.DeviceBatch(b, scorer=scorer)
    d.round()
    torch.cuda.synchronize()
    ora = oracle.round_(b)
    got = {k: d.host(k) for k in ("bound", "alive", "assign", "cent", "counts", "objective", "Ncs", "mu",
                                  "ucb", "sel")}
    np.testing.assert_array_equal(got["bound"].view(np.uint32), ora.bound.view(np.uint32))
    np.testing.assert_array_equal(got["alive"], ora.alive)
    clean = ora.dirty == 0
    assert clean.sum() >= b.G - 3, f"D={D}: only {clean.sum()} of {b.G} searches without a near-tie"
    cp = clean[search_of(b.seg_off)]
    ck = np.repeat(clean, np.diff(b.koff))
    np.testing.assert_array_equal(got["assign"][cp], ora.assign[cp])
    np.testing.assert_array_equal(got["counts"][ck], ora.counts[ck])
    assert_cent_close(got["cent"][ck], ora.cent[ck], f"D={D}")
    assert_rel_close(got["objective"][clean], ora.objective[clean], what=f"D={D} objective")
    np.testing.assert_array_equal(got["Ncs"][ck], ora.Ncs[ck])
    assert_rel_close(got["mu"][ck], ora.mu[ck], what="mu")
    assert_rel_close(got["ucb"][ck], ora.ucb[ck], what="ucb")
    ok = clean & (ora.near == 0)
    np.testing.assert_array_equal(got["sel"][ok], ora.sel[ok])
    # every search, clean or not: the sizes add up and every cluster index is in range
    assert got["counts"].sum() == b.N
    kg = np.diff(b.koff)[search_of(b.seg_off)]
    assert ((got["assign"] >= 0) & (got["assign"] < kg)).all()


# cluster counts of the multi-workgroup path: one to four centroid groups of 64, whole
# and partly filled
BIG_KS = (65, 100, 128, 129, 192, 193, 255, 256)


def _big_batch(D, seed):
    rng = np.random.default_rng(seed)
    b = None
    for i, K in enumerate(BIG_KS):
        n = int(rng.integers(4 * K + 1, 12 * K))
        one = synth.config2(seed=seed * 100 + i, N=n, D=D, K=K, S=4, iters=4)
        b = one if b is None else synth.concat(b, one, f"sweepbigD{D}")
    return b


@pytest.mark.parametrize("D", [4, 6, 20, 36, 48, 64])
@pytest.mark.parametrize("scorer", [0, 1], ids=["matrixcore", "vectoralu"])
def test_multi_workgroup_clustering_over_shapes(kb, D, scorer):
    import torch
    b = _big_batch(D, seed=2000 + D)
    d = kb.DeviceBatch(b, scorer=scorer)
    d.cluster()
    torch.cuda.synchronize()
    ora = oracle.cluster(b.seg_off, b.koff, b.X, b.iters)
    got = {k: d.host(k) for k in ("assign", "cent", "counts", "objective")}
    clean = ora.dirty == 0
    assert clean.sum() >= b.G - 3, f"D={D}: only {clean.sum()} of {b.G} searches without a near-tie"
    cp = clean[search_of(b.seg_off)]
    ck = np.repeat(clean, np.diff(b.koff))
    np.testing.assert_array_equal(got["assign"][cp], ora.assign[cp])
    np.testing.assert_array_equal(got["counts"][ck], ora.counts[ck])
    assert_cent_close(got["cent"][ck], ora.cent[ck], f"D={D}")
    assert_rel_close(got["objective"][clean], ora.objective[clean], what=f"D={D} objective")
    assert got["counts"].sum() == b.N


# strategy counts of every row form of the selection kernels: 16-byte pieces in a power
# of two per row (4, 8), 16-byte pieces otherwise (12, 20, 24), 8-byte pieces (2, 6, 10),
# single values (1, 5, 7)
@pytest.mark.parametrize("S", [1, 2, 4, 5, 6, 7, 8, 10, 12, 20, 24])
def test_selection_over_strategy_counts(kb, S):
    """The selection step against the oracle for each S: 40 searches of 64-3000 candidates
    (one workgroup each), one of 20000 behind them (candidate ranges and global tables), and
    the same 40 alone shortened to at most 200 candidates (a wave each)."""
    import torch
    short = synth.config5(G=40, nmin=20, nmax=200, D=8, S=S, iters=2, seed=300 + S)
    mid = synth.config5(G=40, nmin=64, nmax=3000, D=8, S=S, iters=2, seed=400 + S)
    both = synth.concat(mid, synth.config2(N=20000, D=8, K=6, S=S, iters=2, seed=500 + S), f"S{S}")
    for b in (short, mid, both):
        bound, alive = oracle.prune(b.seg_off, b.flops, b.bytes_, b.peak_flops, b.peak_bw, b.incumbent)
        cl = oracle.cluster(b.seg_off, b.koff, b.X, 2)
        d = kb.DeviceBatch(b)
        d.assign.copy_(torch.from_numpy(cl.assign))
        d.alive.copy_(torch.from_numpy(alive))
        d.bound.copy_(torch.from_numpy(bound))
        d.ucb_select()
        torch.cuda.synchronize()
        ora = oracle.ucb_select(b.seg_off, b.koff, b.S, cl.assign, alive, bound, b.visits, b.rsum,
                                b.t, b.c, b.prior_n, b.prior_mu)
        np.testing.assert_array_equal(d.host("Ncs"), ora.Ncs, err_msg=f"S={S} {b.name}")
        assert_rel_close(d.host("mu"), ora.mu, what=f"S={S} mu")
        assert_rel_close(d.host("ucb"), ora.ucb, what=f"S={S} ucb")
        ok = ora.near == 0
        assert ok.sum() >= b.G - 2
        np.testing.assert_array_equal(d.host("sel")[ok], ora.sel[ok], err_msg=f"S={S} {b.name}")
