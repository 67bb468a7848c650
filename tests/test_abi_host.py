"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/kb.h declares, and rejects bad arguments before touching
the device."""
import ctypes
import os
import re

import pytest

from paper_2511_18868_amd import binding as kb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000   # non-NULL, 256-byte aligned; never dereferenced on these paths


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(kb.LIB_PATH):
        from paper_2511_18868_amd import build
        build.build()
    return kb.lib()


def test_exports_every_declared_symbol(L):
    hdr = open(os.path.join(ROOT, "include", "kb.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(kb_[a-z_]+)\s*\(", hdr))
    assert {"kb_prune", "kb_cluster_step", "kb_cluster", "kb_ucb_select", "kb_round",
            "kb_workspace_bytes", "kb_status_str", "kb_version", "kb_sample"} <= names
    for n in names:
        assert hasattr(L, n), n


def test_struct_layout_matches_header():
    assert ctypes.sizeof(kb.kb_batch) == 56
    assert ctypes.sizeof(kb.kb_params) == 32 and kb.kb_params.scorer.offset == 24
    assert kb.kb_params.stop_early.offset == 28
    assert ctypes.sizeof(kb.kb_round_io) == 17 * 8
    assert kb.kb_batch.N.offset == 16 and kb.kb_batch.seg_off.offset == 40


def _batch(G=2, D=8, S=4, N=100, Kmax=4, Ksum=8, Nmax=60, seg=FAKE, ko=FAKE):
    return kb.make_batch(G, D, S, N, Kmax, Ksum, Nmax, seg, ko)


def test_status_strings(L):
    for s in range(5):
        assert L.kb_status_str(s).decode().startswith("KB_")
    assert "unknown" in L.kb_status_str(99).decode()
    assert kb.kb_version()


def test_workspace_bytes_is_pure_and_monotone(L):
    p = kb.make_params()
    a = kb.kb_workspace_bytes(_batch(N=100, Nmax=60), p)
    b = kb.kb_workspace_bytes(_batch(N=100000, Nmax=60), p)
    assert 0 < a < b and a % 256 == 0
    assert kb.kb_workspace_bytes(_batch(G=0), p) == 0


@pytest.mark.parametrize("bad", [
    dict(G=0), dict(D=0), dict(S=0), dict(N=-1), dict(seg=None), dict(ko=None),
    dict(Kmax=70, Nmax=60), dict(Nmax=200, N=100), dict(Kmax=9, Ksum=8),
])
def test_bad_batch_is_einval(L, bad):
    p = kb.make_params()
    s = kb.kb_prune(_batch(**bad), p, FAKE, FAKE, FAKE, FAKE, FAKE, stream=0, check=False)
    assert s == kb.KB_EINVAL


def test_prune_argument_errors(L):
    b = _batch()
    ok = kb.make_params()
    assert kb.kb_prune(b, ok, None, FAKE, FAKE, FAKE, FAKE, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_prune(b, ok, FAKE, FAKE, FAKE, FAKE, None, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_prune(b, ok, FAKE + 4, FAKE, FAKE, FAKE, FAKE, stream=0, check=False) == kb.KB_EINVAL
    for bad in (dict(peak_flops=0.0), dict(peak_bw=-1.0), dict(peak_flops=float("nan"))):
        assert kb.kb_prune(b, kb.make_params(**bad), FAKE, FAKE, FAKE, FAKE, FAKE, stream=0,
                           check=False) == kb.KB_EINVAL


def test_cluster_argument_errors(L):
    b = _batch()
    p = kb.make_params(iters=3)
    big = 1 << 20
    # workspace missing / misaligned / too small
    assert kb.kb_cluster(b, p, FAKE, None, FAKE, FAKE, FAKE, FAKE, None, big, stream=0,
                         check=False) == kb.KB_EWORKSPACE
    assert kb.kb_cluster(b, p, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE + 16, big, stream=0,
                         check=False) == kb.KB_EWORKSPACE
    assert kb.kb_cluster(b, p, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, 8, stream=0,
                         check=False) == kb.KB_EWORKSPACE
    # NULL X, negative iters, overlapping centroid arrays, missing cent_in for a step
    assert kb.kb_cluster(b, p, None, None, FAKE, FAKE, FAKE, FAKE, FAKE, big, stream=0,
                         check=False) == kb.KB_EINVAL
    assert kb.kb_cluster(b, kb.make_params(iters=-1), FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE,
                         big, stream=0, check=False) == kb.KB_EINVAL
    # stop_early is 0 or 1
    assert kb.kb_cluster(b, kb.make_params(iters=3, stop_early=2), FAKE, None, FAKE, FAKE, FAKE, FAKE,
                         FAKE, big, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_cluster(b, p, FAKE, 0x2000, FAKE, 0x2000 + 16, FAKE, FAKE, FAKE, big, stream=0,
                         check=False) == kb.KB_EINVAL
    assert kb.kb_cluster_step(b, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, big, stream=0,
                              check=False) == kb.KB_EINVAL
    # beyond the compiled limits
    assert kb.kb_cluster(_batch(D=65), p, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, big, stream=0,
                         check=False) == kb.KB_EUNSUPPORTED
    assert kb.kb_cluster(_batch(Kmax=257, Ksum=300, Nmax=400, N=1000), p, FAKE, None, FAKE, FAKE,
                         FAKE, FAKE, FAKE, big, stream=0, check=False) == kb.KB_EUNSUPPORTED


def test_ucb_and_round_argument_errors(L):
    b = _batch()
    p = kb.make_params(iters=2)
    big = 1 << 20
    args = [FAKE] * 10
    bad = list(args)
    bad[3] = None
    assert kb.kb_ucb_select(b, p, *bad, FAKE, big, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_ucb_select(b, kb.make_params(prior_n=-1.0), *args, FAKE, big, stream=0,
                            check=False) == kb.KB_EINVAL
    assert kb.kb_ucb_select(_batch(S=4096, Kmax=4), p, *args, FAKE, big, stream=0,
                            check=False) == kb.KB_EUNSUPPORTED
    io = kb.kb_round_io(*([FAKE] * 17))
    assert kb.kb_round(b, kb.make_params(iters=0), io, FAKE, big, stream=0,
                       check=False) == kb.KB_EINVAL
    io2 = kb.kb_round_io(*([FAKE] * 17))
    io2.sel = None
    assert kb.kb_round(b, p, io2, FAKE, big, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_round(b, p, io, FAKE, 16, stream=0, check=False) == kb.KB_EWORKSPACE


def test_static_selection_rejects_sizes_beyond_its_scratch(L):
    p = kb.make_params(iters=2)
    args = [FAKE] * 10
    assert kb.kb_ucb_select_static(_batch(G=65537, N=1 << 20, Ksum=65537 * 2), p, *args, stream=0,
                                   check=False) == kb.KB_EUNSUPPORTED
    # searches longer than 16384 candidates also need their cluster-arm tables to fit
    assert kb.kb_ucb_select_static(_batch(N=1 << 22, Nmax=20000, Kmax=64, Ksum=70000), p, *args,
                                   stream=0, check=False) == kb.KB_EUNSUPPORTED
    assert kb.kb_ucb_select_static(_batch(N=1 << 22, Nmax=20000, Kmax=64, Ksum=40000, S=4), p, *args,
                                   stream=0, check=False) == kb.KB_EUNSUPPORTED
    bad = list(args)
    bad[0] = None
    assert kb.kb_ucb_select_static(_batch(), p, *bad, stream=0, check=False) == kb.KB_EINVAL


def test_sample_argument_errors(L):
    b = _batch()
    big = 1 << 20
    ok = kb.kb_sample_params(1, 2, 1.0)
    args = [FAKE] * 6      # assign, alive, bound, incumbent, sel, ksel
    for i in (0, 2, 3, 4, 5):
        bad = list(args)
        bad[i] = None
        assert kb.kb_sample(b, ok, *bad, FAKE, big, stream=0, check=False) == kb.KB_EINVAL
    for tau in (0.0, -1.0, float("inf"), float("nan")):
        assert kb.kb_sample(b, kb.kb_sample_params(1, 2, tau), *args, FAKE, big, stream=0,
                            check=False) == kb.KB_EINVAL
    assert kb.kb_sample(b, ok, *args, FAKE, 16, stream=0, check=False) == kb.KB_EWORKSPACE
    assert kb.kb_sample(b, ok, *args, None, big, stream=0, check=False) == kb.KB_EWORKSPACE
    assert ctypes.sizeof(kb.kb_sample_params) == 24


def test_loop_entry_points_argument_errors(L):
    b = _batch()
    p = kb.make_params()
    big = 1 << 20
    sp = kb.kb_sample_params(1, 2, 1.0)
    # geometry: X, cent, assign, rep, radius
    g = [FAKE] * 5
    for i in range(5):
        bad = list(g); bad[i] = None
        assert kb.kb_cluster_geometry(b, *bad, FAKE, big, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_cluster_geometry(b, FAKE + 4, *g[1:], FAKE, big, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_cluster_geometry(b, *g, FAKE, 16, stream=0, check=False) == kb.KB_EWORKSPACE
    assert kb.kb_cluster_geometry(_batch(D=65), *g, FAKE, big, stream=0, check=False) == kb.KB_EUNSUPPORTED
    # mask: R, h, target, rep, theta, M, nvalid
    assert kb.kb_strategy_mask(b, 0, FAKE, FAKE, FAKE, 0.75, FAKE, FAKE, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_strategy_mask(b, 3, None, FAKE, FAKE, 0.75, FAKE, FAKE, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_strategy_mask(b, 3, FAKE, FAKE, FAKE, float("nan"), FAKE, FAKE, stream=0,
                               check=False) == kb.KB_EINVAL
    # masked selection: alive, bound and M may be NULL, the rest may not
    args = [FAKE] * 11
    bad = list(args); bad[0] = None
    assert kb.kb_ucb_select_masked(b, p, *bad, FAKE, big, stream=0, check=False) == kb.KB_EINVAL
    bad = list(args); bad[4] = None
    assert kb.kb_ucb_select_masked(b, p, *bad, FAKE, big, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_ucb_select_masked(b, p, *args, FAKE, 16, stream=0, check=False) == kb.KB_EWORKSPACE
    # update: sel, ksel, reward, ok, visits, rsum, Ncs, mu, t
    u = [FAKE] * 9
    for i in range(9):
        bad = list(u); bad[i] = None
        assert kb.kb_update_stats(b, p, *bad, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_update_stats(b, kb.make_params(prior_n=-1.0), *u, stream=0, check=False) == kb.KB_EINVAL
    # diameters: X, assign, diam
    assert kb.kb_cluster_diameter(b, None, FAKE, FAKE, FAKE, big, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_cluster_diameter(b, FAKE, FAKE, None, FAKE, big, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_cluster_diameter(b, FAKE, FAKE, FAKE, FAKE, 16, stream=0, check=False) == kb.KB_EWORKSPACE
    # farthest-point seeds: X, cent, pick (pick may be NULL)
    assert kb.kb_seed_farthest(b, None, FAKE, FAKE, FAKE, big, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_seed_farthest(b, FAKE, None, FAKE, FAKE, big, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_seed_farthest(b, FAKE, FAKE + 8, None, FAKE, big, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_seed_farthest(b, FAKE, FAKE, None, FAKE, 16, stream=0, check=False) == kb.KB_EWORKSPACE
    assert kb.kb_seed_farthest(_batch(D=65), FAKE, FAKE, None, FAKE, big, stream=0,
                               check=False) == kb.KB_EUNSUPPORTED
    assert kb.kb_seed_dsquared(b, None, 1, 2, FAKE, FAKE, FAKE, big, stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_seed_dsquared(b, FAKE, 1, 2, FAKE, None, FAKE, 16, stream=0, check=False) == kb.KB_EWORKSPACE
    # signature draw
    assert kb.kb_sample_signature(b, sp, FAKE, None, 0, FAKE, FAKE, 0.75, FAKE, FAKE, FAKE, big,
                                  stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_sample_signature(b, sp, FAKE, None, 3, None, FAKE, 0.75, FAKE, FAKE, FAKE, big,
                                  stream=0, check=False) == kb.KB_EINVAL
    assert kb.kb_sample_signature(b, kb.kb_sample_params(1, 2, 0.0), FAKE, None, 3, FAKE, FAKE, 0.75,
                                  FAKE, FAKE, FAKE, big, stream=0, check=False) == kb.KB_EINVAL


def test_scorer_mode_is_validated(L):
    """The scorer mode travels in kb_params (the library keeps no state); a value
    outside KB_SCORER_* is rejected before anything is enqueued."""
    assert not hasattr(L, "kb_set_scorer")
    b = _batch()
    big = 1 << 20
    io = kb.kb_round_io(*([FAKE] * 17))
    for bad in (-1, 3, 7):
        p = kb.make_params(iters=2, scorer=bad)
        assert kb.kb_cluster(b, p, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, big, stream=0,
                             check=False) == kb.KB_EINVAL
        assert kb.kb_round(b, p, io, FAKE, big, stream=0, check=False) == kb.KB_EINVAL


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(kb, "_lib", None)
    monkeypatch.setattr(kb, "LIB_PATH", "/nonexistent/libkernelband.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        kb.lib()
