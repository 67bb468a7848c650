"""kb_iterate - whole iterations of Alg. 1 enqueued in one call - against the
oracle's composition of the same stages, round by round.  A search is compared
up to the first round in which the oracle saw a near-tie in any stage (after
that both sides may legitimately continue differently)."""
import numpy as np
import pytest

import oracle
from paper_2511_18868_amd import synth
from kbcheck import assert_cent_close, assert_rel_close, search_of

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kb():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2511_18868_amd import binding
    binding.lib()
    return binding


def _guarded():
    """config-5-like searches, one of them with more than N/2 clusters (never re-clustered)."""
    b = synth.config5(G=40, nmin=64, nmax=500, S=8, seed=51)
    kg, ng = np.diff(b.koff).copy(), np.diff(b.seg_off)
    kg[3] = ng[3] // 2 + 1
    b.koff = np.concatenate([[0], np.cumsum(kg)]).astype(np.int32)
    return b


def _with_long_search():
    """A search of 20000 candidates (its cluster-arm tables are aggregated over candidate
    ranges) after 30 short ones."""
    a = synth.config5(G=30, nmin=64, nmax=500, D=16, S=4, iters=2, seed=54)
    big = synth.config2(N=20000, D=16, K=8, S=4, iters=2, seed=6)
    return synth.concat(a, big, "longsearch")


CASES = {
    # name: (batch, rounds, tau, t0, warm_start, Lloyd steps per re-clustering)
    "paper": (lambda: synth.paper_shape(), 25, 10, 0, 0, 5),
    "cfg5s": (lambda: synth.config5(G=64, nmin=64, nmax=700, S=8, seed=50), 30, 10, 0, 1, 2),
    "guard": (_guarded, 26, 5, 2, 1, 2),
    "multiworkgroup": (lambda: synth.config5(G=4, nmin=1500, nmax=4000, kcap=128, D=40, S=4, iters=3,
                                             seed=52), 7, 3, 0, 1, 2),
    "never": (lambda: synth.config3(G=16), 12, 0, 5, 0, 1),
    "longsearch": (_with_long_search, 14, 6, 0, 1, 2),
    # with a mask of alive candidates (every third one pruned)
    "pruned": (lambda: synth.config5(G=24, nmin=64, nmax=400, S=8, seed=55), 22, 8, 1, 1, 2),
    # short searches only: clustering, representatives and draw run a wave per search
    "paperscale": (lambda: synth.paper_scale(), 24, 6, 0, 1, 4),
    "short": (lambda: synth.config5(G=120, nmin=8, nmax=256, D=12, S=4, kcap=16, kdiv=4, seed=78), 18, 5, 1, 0, 3),
}


@pytest.mark.parametrize("name", list(CASES))
def test_iterate_matches_the_composed_oracle(kb, name):
    import torch
    make, T, tau, t0, warm, iters = CASES[name]
    b = make()
    R = 3
    h, target, theta = synth.signatures(b, R)
    fb = [synth.feedback(b, seed=r) for r in range(T)]
    rw, ok = np.stack([f[0] for f in fb]), np.stack([f[1] for f in fb])
    seed, draw0, temp = 20251118, 100, 1.0

    # common starting state: two Lloyd steps, representatives, mask (from the oracle)
    cl = oracle.cluster(b.seg_off, b.koff, b.X, 2)
    geo = oracle.cluster_geometry(b.seg_off, b.koff, b.X, cl.cent, cl.assign)
    M0 = oracle.strategy_mask(b.koff, b.S, h, target, geo.rep, theta).M

    d = kb.DeviceBatch(b, iters=iters)
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(d.device)
    d.assign.copy_(up(cl.assign)); d.cent.copy_(up(cl.cent)); d.counts.copy_(up(cl.counts))
    d.objective.copy_(up(cl.objective.astype(np.float32)))
    d.rep.copy_(up(geo.rep)); d.M.copy_(up(M0))
    dh, dtg, drw, dok = up(h), up(target), up(rw), up(ok)
    sel_log = torch.full((T, b.G, 3), -7, dtype=torch.int32, device=d.device)
    ksel_log = torch.full((T, b.G), -7, dtype=torch.int32, device=d.device)
    ip = kb.kb_iterate_params(T, tau, t0, warm, R, theta, kb.kb_sample_params(seed, draw0, temp))
    alive = None
    if name == "pruned":
        alive = (np.arange(b.N) % 3 != 1).astype(np.uint8)
    d.iterate(ip, dh, dtg, drw, dok, sel_log, ksel_log, alive=None if alive is None else up(alive))
    torch.cuda.synchronize()

    o = oracle.iterate(b.seg_off, b.koff, b.S, b.X, h, target, theta, alive, rw, ok, b.visits, b.rsum,
                       b.t, cl.assign, cl.cent, cl.counts, cl.objective, geo.rep, M0, T, tau, t0, warm,
                       iters, b.c, b.prior_n, b.prior_mu, seed, draw0, temp)
    gs, gk = sel_log.cpu().numpy(), ksel_log.cpu().numpy()
    clean = cl.dirty == 0
    compared = 0
    for r in range(T):
        clean = clean & (o.doubt[r] == 0)
        np.testing.assert_array_equal(gs[r][clean], o.sel_log[r][clean], err_msg=f"{name} sel round {r}")
        np.testing.assert_array_equal(gk[r][clean], o.ksel_log[r][clean], err_msg=f"{name} ksel round {r}")
        compared += int(clean.sum())
    cp = clean[search_of(b.seg_off)]
    ck = np.repeat(clean, np.diff(b.koff))
    np.testing.assert_array_equal(d.host("t"), o.t)                         # every search, clean or not
    np.testing.assert_array_equal(d.host("visits")[cp], o.visits[cp])
    np.testing.assert_array_equal(d.host("rsum")[cp], o.rsum[cp])
    np.testing.assert_array_equal(d.host("assign")[cp], o.assign[cp])
    np.testing.assert_array_equal(d.host("counts")[ck], o.counts[ck])
    assert_cent_close(d.host("cent")[ck], o.cent[ck], name)
    np.testing.assert_array_equal(d.host("rep")[ck], o.rep[ck])
    np.testing.assert_array_equal(d.host("M")[ck], o.M[ck])
    np.testing.assert_array_equal(d.host("Ncs")[ck], o.Ncs[ck])
    assert_rel_close(d.host("mu")[ck], o.mu[ck], what=name + " mu")
    # the selections are valid arms on every search, compared or not
    ng, kg = np.diff(b.seg_off), np.diff(b.koff)
    live = ng > 0
    assert ((gs[:, live, 0] >= 0) & (gs[:, live, 0] < kg[live])).all()
    assert ((gk[:, live] >= b.seg_off[:-1][live]) & (gk[:, live] < b.seg_off[1:][live])).all()
    print(f"[{name}] {T} rounds x {b.G} searches: {compared} search-rounds compared, "
          f"{int(clean.sum())} searches clean to the end", flush=True)
    assert compared >= 0.7 * T * b.G


def test_iterate_argument_errors(kb):
    import torch
    b = synth.config5(G=4, nmin=64, nmax=100, S=4, seed=53)
    d = kb.DeviceBatch(b, iters=1)
    h, target, theta = synth.signatures(b, 3)
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(d.device)
    dh, dtg = up(h), up(target)
    drw, dok = up(np.zeros((2, b.G), np.float32)), up(np.ones((2, b.G), np.uint8))
    sl = torch.zeros((2, b.G, 3), dtype=torch.int32, device=d.device)
    kl = torch.zeros((2, b.G), dtype=torch.int32, device=d.device)
    sp = kb.kb_sample_params(1, 1, 1.0)
    for bad in (kb.kb_iterate_params(0, 10, 0, 0, 3, theta, sp),
                kb.kb_iterate_params(2, 10, -1, 0, 3, theta, sp),
                kb.kb_iterate_params(2, 10, 0, 0, 0, theta, sp),
                kb.kb_iterate_params(2, 10, 0, 0, 3, theta, kb.kb_sample_params(1, 1, 0.0))):
        assert d.iterate(bad, dh, dtg, drw, dok, sl, kl, check=False) == kb.KB_EINVAL
    good = kb.kb_iterate_params(2, 10, 0, 0, 3, theta, sp)
    assert d.iterate(good, None, dtg, drw, dok, sl, kl, check=False) == kb.KB_EINVAL
    assert d.iterate(good, dh, dtg, drw, dok, sl, kl, check=False) == kb.KB_OK
    torch.cuda.synchronize()
