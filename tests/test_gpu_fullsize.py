"""GPU parity at the full sizes of the five benchmark configurations, in the
launch configuration bench.py times (kb_round on the whole batch).

Configurations 1 and 2 are already full size in test_gpu_parity.py.  3 and 5
are compared with the oracle element by element, and so is 4 (one search of
2^20 candidates, 256 clusters), step by step over its ten Lloyd steps."""
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


def _sync():
    import torch
    torch.cuda.synchronize()


# searches the oracle excludes as near-ties at full size (seeded inputs, deterministic
# oracle: exact counts; none of the selections is a near-tie)
NEAR_TIE_SEARCHES = {"config3": 3, "config5": 56, "manytiny": 0}


def _full_round_vs_oracle(kb, b, name):
    d = kb.DeviceBatch(b)
    d.round()
    _sync()
    print(f"[{name}] GPU round done, running the oracle on {b.N} candidates", flush=True)
    ora = oracle.round_(b)
    np.testing.assert_array_equal(d.host("bound").view(np.uint32), ora.bound.view(np.uint32))
    np.testing.assert_array_equal(d.host("alive"), ora.alive)
    clean = ora.dirty == 0
    cp = clean[search_of(b.seg_off)]
    ck = np.repeat(clean, np.diff(b.koff))
    np.testing.assert_array_equal(d.host("assign")[cp], ora.assign[cp])
    np.testing.assert_array_equal(d.host("counts")[ck], ora.counts[ck])
    assert_cent_close(d.host("cent")[ck], ora.cent[ck], name)
    assert_rel_close(d.host("objective")[clean], ora.objective[clean], what=name + " objective")
    np.testing.assert_array_equal(d.host("Ncs")[ck], ora.Ncs[ck])
    assert_rel_close(d.host("mu")[ck], ora.mu[ck], what="mu")
    assert_rel_close(d.host("ucb")[ck], ora.ucb[ck], what="ucb")
    ok = clean & (ora.near == 0)
    np.testing.assert_array_equal(d.host("sel")[ok], ora.sel[ok])
    # searches the oracle saw a near-tie in: still a valid clustering state
    a, cnt = d.host("assign"), d.host("counts")
    for g in np.where(~clean)[0]:
        K = b.koff[g + 1] - b.koff[g]
        np.testing.assert_array_equal(cnt[b.koff[g]:b.koff[g + 1]],
                                      np.bincount(a[b.seg_off[g]:b.seg_off[g + 1]], minlength=K))
    same = sum(np.array_equal(a[b.seg_off[g]:b.seg_off[g + 1]], ora.assign[b.seg_off[g]:b.seg_off[g + 1]])
               for g in np.where(~clean)[0])
    print(f"[{name}] {b.G} searches: {int(clean.sum())} compared bit-exactly, {int((~clean).sum())} "
          f"excluded as near-tie (of which {same} match anyway), {int((ora.near != 0).sum())} "
          f"selections excluded as near-tie", flush=True)
    assert (~clean).sum() <= NEAR_TIE_SEARCHES[name] and (ora.near == 0).all()
    _loop_steps_vs_oracle(kb, b, d, name, ora, ok)


def _loop_steps_vs_oracle(kb, b, d, name, ora=None, ok=None):
    """The in-cluster draw and the cluster representatives at full size, on the
    state the round just left on the device."""
    import torch
    d.sample(20251118, 7, 1.0)
    d.cluster_geometry()
    _sync()
    a, cent = d.host("assign"), d.host("cent")
    alive, bound, sel = d.host("alive"), d.host("bound"), d.host("sel")
    # the draw, given the device's own selection (exact inputs, index output)
    want = oracle.sample(b.seg_off, a, alive, bound, b.incumbent, sel, 20251118, 7, 1.0)
    fine = want.near == 0
    np.testing.assert_array_equal(d.host("ksel")[fine], want.ksel[fine], err_msg=name + " ksel")
    assert fine.mean() > 0.999
    if ora is not None:
        # and end to end against the oracle's own round where nothing was a near-tie
        w2 = oracle.sample(b.seg_off, ora.assign, ora.alive, ora.bound, b.incumbent, ora.sel,
                           20251118, 7, 1.0)
        e2e = ok & (w2.near == 0)
        np.testing.assert_array_equal(d.host("ksel")[e2e], w2.ksel[e2e], err_msg=name + " ksel e2e")
    # representatives and radii of the final clustering: exact on every cluster
    g = oracle.cluster_geometry(b.seg_off, b.koff, b.X, cent, a)
    np.testing.assert_array_equal(d.host("rep"), g.rep, err_msg=name + " rep")
    np.testing.assert_array_equal(d.host("radius"), g.radius.astype(np.float32), err_msg=name + " radius")
    print(f"[{name}] draw compared on {int(fine.sum())} of {b.G} searches, representatives and "
          f"radii exact on {b.Ksum} clusters", flush=True)
    # diameters: all clusters where the pair loop of the oracle is affordable, otherwise
    # a few clusters taken out as searches of their own
    d.cluster_diameter()
    _sync()
    diam = d.host("diam")
    cnt = np.bincount(np.repeat(b.koff[:-1], np.diff(b.seg_off)) + a, minlength=b.Ksum)
    if float((cnt.astype(np.float64) ** 2).sum()) < 5e8:
        assert_rel_close(diam, oracle.cluster_diameter(b.seg_off, b.koff, b.X, a), what=name + " diameter")
        checked = b.Ksum
    else:
        rng = np.random.default_rng(1)
        checked = 0
        for j in rng.choice(b.Ksum, size=3, replace=False):
            g = int(np.searchsorted(b.koff, j, side="right") - 1)
            mem = np.where(a[b.seg_off[g]:b.seg_off[g + 1]] == j - b.koff[g])[0] + b.seg_off[g]
            mem = mem[:6000]          # the diameter of a subset is a lower bound ...
            sub = oracle.cluster_diameter(np.array([0, len(mem)], np.int32), np.array([0, 1], np.int32),
                                          b.X[mem], np.zeros(len(mem), np.int32))[0]
            if len(mem) == cnt[j]:
                assert_rel_close(diam[j:j + 1], np.array([sub]), what=name + " diameter")
                checked += 1
            else:
                assert diam[j] >= sub * (1 - 1e-5)
        # ... and on every cluster: radius <= diameter <= 2 radius
    rad = d.host("radius")
    many = cnt > 1
    assert (diam[many] <= 2 * rad[many] * (1 + 1e-5)).all() and (diam[many] >= rad[many] * (1 - 1e-5)).all()
    print(f"[{name}] diameters compared on {checked} clusters, bracketed by the radii on all", flush=True)


def test_config3_full(kb):
    _full_round_vs_oracle(kb, synth.config3(), "config3")


def test_config5_full(kb):
    _full_round_vs_oracle(kb, synth.config5(), "config5")


def test_many_tiny_searches_full(kb):
    """20000 searches of 1 to 40 candidates: every stage runs its wave-per-search kernel,
    at a grid of 5000 workgroups."""
    _full_round_vs_oracle(kb, synth.config5(G=20000, nmin=1, nmax=40, D=8, S=4, iters=4, seed=15), "manytiny")


def _oracle_assign_sliced(b, cent, parts=64):
    """The oracle's nearest centroid for every candidate of a one-search batch.  The
    rows are handed over as `parts` slices with a copy of the centroids each, which
    the oracle's loop over searches spreads over the host threads."""
    assert b.G == 1
    K = int(b.koff[1])
    seg = np.linspace(0, b.N, parts + 1).astype(np.int32)
    ko = (np.arange(parts + 1) * K).astype(np.int32)
    return oracle.assign(seg, ko, b.X, np.tile(cent, (parts, 1)))


def test_config4_full(kb):
    """One search of 2^20 candidates, 256 clusters, 10 Lloyd steps: every step is
    compared with the oracle on EVERY candidate.  Both sides start each step from the
    same centroids (the device's); where the oracle flags a near-tie the device's
    choice is adopted, everything else must be equal."""
    import torch
    b = synth.config4()
    d = kb.DeviceBatch(b)
    cur = b.X[:b.Ksum].copy()                      # init = first K rows
    prevJ = np.inf
    nflag_total = 0
    for it in range(b.iters):
        d.cluster_step(torch.from_numpy(cur).to(d.device))
        _sync()
        got = {k: d.host(k).copy() for k in ("assign", "cent", "counts", "objective")}
        a_o, mind2, flag = _oracle_assign_sliced(b, cur)
        diff = got["assign"] != a_o
        assert not (diff & (flag == 0)).any(), \
            f"step {it}: {(diff & (flag == 0)).sum()} unflagged assignments differ"
        nflag_total += int(flag.sum())
        adopted = np.where(flag != 0, got["assign"], a_o)
        # flagged candidates: the device's choice is one of the two nearly equal nearest
        for k in np.where(diff)[0]:
            dk = ((b.X[k].astype(np.float64) - cur[got["assign"][k]].astype(np.float64)) ** 2).sum()
            assert dk <= mind2[k] * (1 + 2e-6)
        np.testing.assert_array_equal(got["counts"], np.bincount(adopted, minlength=b.Ksum))
        upd, _ = oracle.update(b.seg_off, b.koff, b.X, cur, adopted)
        assert_cent_close(got["cent"], upd, f"config4 step {it}")
        assert_rel_close(got["objective"], np.array([mind2.sum()]), what=f"config4 step {it} objective")
        assert got["objective"][0] <= prevJ * (1 + 1e-6)
        prevJ = float(got["objective"][0])
        print(f"[config4] step {it}: {b.N} assignments compared, {int(flag.sum())} flagged by the "
              f"oracle, {int(diff.sum())} of those resolved differently", flush=True)
        cur = got["cent"]
    assert nflag_total < 1e-4 * b.N * b.iters
    last = got
    # the fused call and the full round give the bytes of the iterated steps
    d.round()
    _sync()
    for k, v in last.items():
        np.testing.assert_array_equal(d.host(k).view(np.uint8), v.view(np.uint8), err_msg=k)
    bound, alive = oracle.prune(b.seg_off, b.flops, b.bytes_, b.peak_flops, b.peak_bw, b.incumbent)
    np.testing.assert_array_equal(d.host("bound").view(np.uint32), bound.view(np.uint32))
    np.testing.assert_array_equal(d.host("alive"), alive)
    u = oracle.ucb_select(b.seg_off, b.koff, b.S, d.host("assign"), alive, bound, b.visits, b.rsum,
                          b.t, b.c)
    np.testing.assert_array_equal(d.host("Ncs"), u.Ncs)
    assert_rel_close(d.host("mu"), u.mu, what="mu")
    assert_rel_close(d.host("ucb"), u.ucb, what="ucb")
    if not u.near[0]:
        np.testing.assert_array_equal(d.host("sel"), u.sel)
    # determinism of the multi-workgroup path
    first = {k: d.host(k).copy() for k in ("assign", "cent", "counts", "objective", "sel")}
    d.round()
    _sync()
    for k, v in first.items():
        np.testing.assert_array_equal(d.host(k).view(np.uint8), v.view(np.uint8), err_msg=k)
    # the fp32 vector-ALU scorer reaches the same bytes
    dv = kb.DeviceBatch(b, scorer=kb.KB_SCORER_VECTOR_ALU)
    dv.cluster()
    _sync()
    for k in ("assign", "cent", "counts", "objective"):
        np.testing.assert_array_equal(dv.host(k).view(np.uint8), first[k].view(np.uint8), err_msg=k)
    del dv
    _loop_steps_vs_oracle(kb, b, d, "config4")
