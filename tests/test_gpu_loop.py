"""GPU parity of the steps that close the loop of Alg. 1 around the scoring pass
- cluster representatives and radii, the strategy mask in the paper's own form,
selection under that mask, the draw with the paper's potential and the statistics
update - against the CPU oracle, through the C ABI.  Indices, masks and counts
are compared bit-exactly; the distances behind the representatives are formed in
the same precision and order on both sides, so they need no exclusions."""
import numpy as np
import pytest

import oracle
from paper_2511_18868_amd import synth
from kbcheck import assert_rel_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kb():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2511_18868_amd import binding
    binding.lib()
    return binding


def _sync():
    import torch
    torch.cuda.synchronize()


def _up(d, a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to(d.device)


def _with_empty_searches():
    b = synth.config5(G=12, nmin=64, nmax=200, seed=8)
    ng = np.diff(b.seg_off); kg = np.diff(b.koff)
    ins = [0, 5, len(ng)]
    ng2 = np.insert(ng, ins, 0); kg2 = np.insert(kg, ins, 0)
    b.seg_off = np.concatenate([[0], np.cumsum(ng2)]).astype(np.int32)
    b.koff = np.concatenate([[0], np.cumsum(kg2)]).astype(np.int32)
    b.G = len(ng2)
    b.incumbent = np.insert(b.incumbent, ins, 1.0).astype(np.float32)
    b.t = np.insert(b.t, ins, 1).astype(np.int64)
    return b


CASES = {
    "cfg1": lambda: synth.config1(),
    "cfg2": lambda: synth.config2(),
    "cfg3s": lambda: synth.config3(G=48),
    "cfg5s": lambda: synth.config5(G=96),
    "paper": lambda: synth.paper_shape(),                       # D = 5: the scalar row path
    "ragged": lambda: synth.config5(G=17, nmin=64, nmax=700, D=20, S=6, seed=99),
    "oddD": lambda: synth.config5(G=9, nmin=64, nmax=900, D=7, S=3, seed=4),
    "empty": _with_empty_searches,
    "cfg4s": lambda: synth.config4(N=8192, K=256, ncentres=256),  # largest LDS footprint
    "bigN": lambda: synth.config2(N=70001, D=16, K=8, S=4, iters=2, seed=5),
    # batches of short searches (at most 256 candidates each): a wave per search in the
    # representative pass and the draw
    "paperscale": lambda: synth.paper_scale(),
    "short": lambda: synth.config5(G=300, nmin=1, nmax=256, D=12, S=4, iters=3, kcap=16, kdiv=4, seed=77),
    # a longer search behind 300 of the paper's size: waves for the short ones, the range
    # kernels - which skip the short searches of their ranges 64 at a time - for the long one
    "tinylong": lambda: synth.concat(synth.config5(G=300, nmin=12, nmax=41, D=5, S=6, iters=3, kcap=3, kdiv=4,
                                                   seed=21),
                                     synth.config2(N=9000, D=5, K=3, S=6, iters=3, seed=22), "tinylong"),
}


@pytest.fixture(scope="module", params=list(CASES))
def case(request):
    b = CASES[request.param]()
    c = oracle.cluster(b.seg_off, b.koff, b.X, min(b.iters, 3))
    return request.param, b, c


def test_cluster_geometry_exact(kb, case):
    name, b, c = case
    d = kb.DeviceBatch(b)
    d.assign.copy_(_up(d, c.assign))
    d.cent.copy_(_up(d, c.cent))
    d.rep.fill_(-5)
    d.radius.fill_(-1.0)
    d.cluster_geometry()
    _sync()
    want = oracle.cluster_geometry(b.seg_off, b.koff, b.X, c.cent, c.assign)
    np.testing.assert_array_equal(d.host("rep"), want.rep, err_msg=name)
    np.testing.assert_array_equal(d.host("radius"), want.radius.astype(np.float32), err_msg=name)
    # an empty cluster (when the case has one) reports -1 / 0
    empty = c.counts == 0
    assert (d.host("rep")[empty] == -1).all() and (d.host("radius")[empty] == 0).all()
    # twice in a row on the same workspace: same bytes
    d.cluster_geometry()
    _sync()
    np.testing.assert_array_equal(d.host("rep"), want.rep)


def test_geometry_ties_and_duplicates(kb):
    # duplicate rows at the minimum distance: the lowest index is the representative
    b = synth.config5(G=4, nmin=100, nmax=300, seed=13)
    c = oracle.cluster(b.seg_off, b.koff, b.X, 3)
    g = oracle.cluster_geometry(b.seg_off, b.koff, b.X, c.cent, c.assign)
    X = b.X.copy()
    assign = c.assign.copy()
    moved = 0
    for s in range(b.G):
        for j in range(b.koff[s], b.koff[s + 1]):
            r = g.rep[j]
            mem = np.where(assign[b.seg_off[s]:b.seg_off[s + 1]] == j - b.koff[s])[0] + b.seg_off[s]
            later = mem[mem > r]
            earlier = mem[mem < r]
            if len(later) and len(earlier):
                X[later[-1]] = X[r]          # a copy of the representative after it
                X[earlier[0]] = X[r]         # and one before it: that one must win
                moved += 1
    assert moved > 10
    b.X = X
    d = kb.DeviceBatch(b)
    d.assign.copy_(_up(d, assign))
    d.cent.copy_(_up(d, c.cent))
    d.cluster_geometry()
    _sync()
    want = oracle.cluster_geometry(b.seg_off, b.koff, X, c.cent, assign)
    assert (want.rep != g.rep).sum() >= moved
    np.testing.assert_array_equal(d.host("rep"), want.rep)
    np.testing.assert_array_equal(d.host("radius"), want.radius.astype(np.float32))


def test_mask_selection_draw_update_chain(kb, case):
    """The paper-form iteration on identical inputs, step by step."""
    import torch
    name, b, c = case
    R = 3
    h, target, theta = synth.signatures(b, R)
    g = oracle.cluster_geometry(b.seg_off, b.koff, b.X, c.cent, c.assign)
    d = kb.DeviceBatch(b)
    d.assign.copy_(_up(d, c.assign))
    dh, dt, drep = _up(d, h), _up(d, target), _up(d, g.rep)
    # mask
    kb.kb_strategy_mask(d.batch, R, dh, dt, drep, theta, d.M, d.nvalid)
    _sync()
    m = oracle.strategy_mask(b.koff, b.S, h, target, g.rep, theta)
    np.testing.assert_array_equal(d.host("M"), m.M)
    np.testing.assert_array_equal(d.host("nvalid"), m.nvalid)
    assert 0 < m.M.mean() < 1
    # selection under the mask, every candidate alive, no bounds
    kb.kb_ucb_select_masked(d.batch, d.params, d.assign, None, None, d.M, d.visits, d.rsum, d.t,
                            d.Ncs, d.mu, d.ucb, d.sel, d.ws, d.ws_bytes)
    _sync()
    u = oracle.ucb_select(b.seg_off, b.koff, b.S, c.assign, None, None, b.visits, b.rsum, b.t, b.c,
                          b.prior_n, b.prior_mu, M=m.M)
    np.testing.assert_array_equal(d.host("Ncs"), u.Ncs)
    assert_rel_close(d.host("mu"), u.mu, what="mu")
    assert_rel_close(d.host("ucb"), u.ucb, what="ucb")
    ok = u.near == 0
    np.testing.assert_array_equal(d.host("sel")[ok], u.sel[ok])
    assert np.isneginf(d.host("ucb")[m.M == 0]).all()
    # the draw with V = theta - h[k, target[S*]] on the oracle's selection
    d.sel.copy_(_up(d, u.sel))
    sp = kb.kb_sample_params(11, 3, 0.1)
    kb.kb_sample_signature(d.batch, sp, d.assign, None, R, dh, dt, theta, d.sel, d.ksel, d.ws,
                           d.ws_bytes)
    _sync()
    s = oracle.sample_signature(b.seg_off, c.assign, None, h, target, theta, u.sel, 11, 3,
                                float(np.float32(0.1)))
    oks = s.near == 0
    np.testing.assert_array_equal(d.host("ksel")[oks], s.ksel[oks])
    # the update, in place, from the oracle's tables so that both start equal
    reward, okv = synth.feedback(b)
    Ncs0 = u.Ncs.astype(np.int32)
    mu0 = np.nan_to_num(u.mu.astype(np.float32), nan=0.5)
    d.Ncs.copy_(_up(d, Ncs0)); d.mu.copy_(_up(d, mu0)); d.ksel.copy_(_up(d, s.ksel))
    kb.kb_update_stats(d.batch, d.params, d.sel, d.ksel, _up(d, reward), _up(d, okv), d.visits,
                       d.rsum, d.Ncs, d.mu, d.t)
    _sync()
    w = oracle.update_stats(b.koff, b.S, u.sel, s.ksel, reward, okv, b.prior_n, b.visits, b.rsum,
                            Ncs0, mu0, b.t)
    np.testing.assert_array_equal(d.host("visits"), w.visits)
    np.testing.assert_array_equal(d.host("Ncs"), w.Ncs)
    np.testing.assert_array_equal(d.host("t"), w.t)
    np.testing.assert_array_equal(d.host("rsum").view(np.uint32), w.rsum.view(np.uint32))
    np.testing.assert_array_equal(d.host("mu").view(np.uint32), w.mu.view(np.uint32))
    changed = (w.Ncs != Ncs0).sum()
    assert changed == int(((okv != 0) & (u.sel[:, 0] >= 0) & (s.ksel >= 0)).sum())


def test_masked_selection_reduces_to_plain_selection(kb):
    b = synth.config5(G=40, nmin=64, nmax=2000, seed=3)
    ora = oracle.round_(b, iters=2)
    d = kb.DeviceBatch(b)
    for n in ("assign", "alive", "bound"):
        getattr(d, n).copy_(_up(d, getattr(ora, n)))
    d.ucb_select()
    _sync()
    plain = {k: d.host(k).copy() for k in ("Ncs", "mu", "ucb", "sel")}
    d.M.fill_(1)
    for M in (None, d.M):
        d.sel.fill_(-9)
        kb.kb_ucb_select_masked(d.batch, d.params, d.assign, d.alive, d.bound, M, d.visits, d.rsum,
                                d.t, d.Ncs, d.mu, d.ucb, d.sel, d.ws, d.ws_bytes)
        _sync()
        for k, v in plain.items():
            np.testing.assert_array_equal(d.host(k).view(np.uint8), v.view(np.uint8), err_msg=k)
    d.M.fill_(0)
    kb.kb_ucb_select_masked(d.batch, d.params, d.assign, d.alive, d.bound, d.M, d.visits, d.rsum,
                            d.t, d.Ncs, d.mu, d.ucb, d.sel, d.ws, d.ws_bytes)
    _sync()
    assert (d.host("sel") == -1).all()


def test_seed_farthest_exact(kb, case):
    name, b, _ = case
    d = kb.DeviceBatch(b)
    d.cent2.fill_(-3.0)
    d.rep.fill_(-7)
    d.seed_farthest()
    _sync()
    want = oracle.seed_farthest(b.seg_off, b.koff, b.X)
    np.testing.assert_array_equal(d.host("rep"), want.pick, err_msg=name)
    np.testing.assert_array_equal(d.host("cent2").view(np.uint32), want.cent.view(np.uint32), err_msg=name)
    # pick may be NULL
    d.cent2.fill_(-3.0)
    d.seed_farthest(pick=False)
    _sync()
    np.testing.assert_array_equal(d.host("cent2").view(np.uint32), want.cent.view(np.uint32))


def test_clustering_from_farthest_seeds(kb):
    # the seeds feed kb_cluster as cent_init; the result is the oracle's from the same
    # seeds, and its covering radius beats the one reached from the first K rows
    b = synth.config5(G=24, nmin=64, nmax=1500, seed=61)
    d = kb.DeviceBatch(b, iters=5)
    d.seed_farthest()
    d.cluster(cent_init=d.cent2)
    d.cluster_geometry()
    _sync()
    seeds = oracle.seed_farthest(b.seg_off, b.koff, b.X)
    ora = oracle.cluster(b.seg_off, b.koff, b.X, 5, cent_init=seeds.cent)
    clean = ora.dirty == 0
    cp = np.repeat(clean, np.diff(b.seg_off))
    np.testing.assert_array_equal(d.host("assign")[cp], ora.assign[cp])
    assert clean.mean() > 0.8
    r_far = d.host("radius").copy()
    d.cluster()
    d.cluster_geometry()
    _sync()
    r_first = d.host("radius")
    worst = lambda r: np.array([r[b.koff[g]:b.koff[g + 1]].max() for g in range(b.G)])
    assert (worst(r_far) <= worst(r_first)).mean() > 0.7


def test_batch_without_candidates(kb):
    """Every search empty (N = 0): each entry point returns without touching memory it
    does not own and reports 'nothing' where it reports at all."""
    import torch
    dev = torch.device("cuda:0")
    G, D, S = 3, 8, 4
    z = lambda n, dt: torch.zeros(max(n, 1), dtype=dt, device=dev)
    seg = torch.zeros(G + 1, dtype=torch.int32, device=dev)
    ko = torch.zeros(G + 1, dtype=torch.int32, device=dev)
    batch = kb.make_batch(G, D, S, 0, 0, 0, 0, seg, ko)
    params = kb.make_params(iters=3)
    wsb = kb.kb_workspace_bytes(batch, params)
    assert wsb > 0
    ws = z(wsb, torch.uint8)
    X, cent = z(4, torch.float32), z(4, torch.float32)
    f32, i32, u8 = z(4, torch.float32), z(4, torch.int32), z(4, torch.uint8)
    inc = torch.ones(G, dtype=torch.float32, device=dev)
    t = torch.ones(G, dtype=torch.int64, device=dev)
    sel = torch.full((G, 3), 5, dtype=torch.int32, device=dev)
    ksel = torch.full((G,), 5, dtype=torch.int32, device=dev)
    nvalid = torch.full((G,), 5, dtype=torch.int32, device=dev)
    obj = torch.full((G,), -1.0, dtype=torch.float32, device=dev)
    assert kb.kb_prune(batch, params, f32, f32, inc, f32, u8) == 0
    assert kb.kb_cluster(batch, params, X, None, i32, cent, i32, obj, ws, wsb) == 0
    assert kb.kb_ucb_select(batch, params, i32, u8, f32, i32, f32, t, i32, f32, f32, sel, ws, wsb) == 0
    assert kb.kb_sample(batch, kb.kb_sample_params(1, 1, 1.0), i32, u8, f32, inc, sel, ksel, ws, wsb) == 0
    assert kb.kb_cluster_geometry(batch, X, cent, i32, i32, f32, ws, wsb) == 0
    assert kb.kb_seed_farthest(batch, X, cent, None, ws, wsb) == 0
    assert kb.kb_strategy_mask(batch, 3, f32, i32, i32, 0.75, u8, nvalid) == 0
    _sync()
    assert (sel.cpu().numpy() == -1).all()
    assert (ksel.cpu().numpy() == -1).all()
    assert (nvalid.cpu().numpy() == 0).all()
    assert (obj.cpu().numpy() == 0).all()


def test_seed_dsquared_matches_oracle(kb, case):
    name, b, _ = case
    d = kb.DeviceBatch(b)
    for seed, draw0 in ((20251118, 0), (3, 2 ** 33 + 5)):
        d.cent2.fill_(-3.0)
        d.rep.fill_(-7)
        d.seed_dsquared(seed, draw0)
        _sync()
        want = oracle.seed_dsquared(b.seg_off, b.koff, b.X, seed, draw0)
        ok = np.repeat(want.near == 0, np.diff(b.koff))
        np.testing.assert_array_equal(d.host("rep")[ok], want.pick[ok], err_msg=name)
        np.testing.assert_array_equal(d.host("cent2")[ok].view(np.uint32), want.cent[ok].view(np.uint32))
        assert ok.mean() > 0.95
        # searches the oracle flagged: still rows of their own search
        pk = d.host("rep")
        sid = np.repeat(np.arange(b.G), np.diff(b.koff))
        assert ((pk >= b.seg_off[sid]) & (pk < b.seg_off[sid + 1])).all()


def test_cluster_diameter(kb, case):
    name, b, c = case
    if name == "bigN":
        # eight clusters of about 9000 members: the oracle's pair loop takes too long here;
        # thinned to every fifth row the structure (members spread over 18 ranges) stays
        keep = np.arange(0, b.N, 5)
        b2 = synth.config2(N=len(keep), D=16, K=8, S=4, iters=2, seed=5)
        b2.X = np.ascontiguousarray(b.X[keep])
        b, c = b2, oracle.cluster(b2.seg_off, b2.koff, b2.X, 2)
    d = kb.DeviceBatch(b)
    d.assign.copy_(_up(d, c.assign))
    d.diam.fill_(-1.0)
    d.cluster_diameter()
    _sync()
    first = d.host("diam").copy()
    want = oracle.cluster_diameter(b.seg_off, b.koff, b.X, c.assign)
    assert_rel_close(first, want, what=name + " diameter")
    assert (first[c.counts < 2] == 0).all()
    # the grouping order varies from run to run, the result does not
    d.cluster_diameter()
    _sync()
    np.testing.assert_array_equal(d.host("diam").view(np.uint32), first.view(np.uint32))


@pytest.mark.parametrize("D", [12, 7, 64])
def test_seeds_of_mixed_search_lengths(kb, D):
    # short searches (one workgroup each, rows in registers, the longer ones partly
    # streamed) next to long ones (one launch per centroid) in one batch, the long
    # ones ending and beginning inside the same candidate range
    b = synth.config5(G=14, nmin=64, nmax=12000, D=D, S=3, seed=5)
    ng = np.diff(b.seg_off)
    assert (ng > 4096).sum() >= 3 and (ng <= 4096).sum() >= 3
    assert ng[0] > 4096 and ng[1] > 4096 and b.seg_off[1] % 1024 != 0
    d = kb.DeviceBatch(b)
    d.cent2.fill_(-3.0)
    d.rep.fill_(-7)
    d.seed_farthest()
    _sync()
    want = oracle.seed_farthest(b.seg_off, b.koff, b.X)
    np.testing.assert_array_equal(d.host("rep"), want.pick)
    np.testing.assert_array_equal(d.host("cent2").view(np.uint32), want.cent.view(np.uint32))
    d.cent2.fill_(-3.0)
    d.rep.fill_(-7)
    d.seed_dsquared(11, 5)
    _sync()
    want = oracle.seed_dsquared(b.seg_off, b.koff, b.X, 11, 5)
    ok = np.repeat(want.near == 0, np.diff(b.koff))
    assert ok.mean() > 0.9
    np.testing.assert_array_equal(d.host("rep")[ok], want.pick[ok])
    np.testing.assert_array_equal(d.host("cent2")[ok].view(np.uint32), want.cent[ok].view(np.uint32))
