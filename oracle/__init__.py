"""ctypes front end of the CPU oracle (kb_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's CPU
baseline leg load this; the product path never does.  Nothing here imports the
GPU package, and the GPU package imports nothing from here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from types import SimpleNamespace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kb_oracle.c")
_LIB = os.path.join(_HERE, "libkb_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile kb_oracle.c with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fopenmp", "-shared",
               "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.kbo_max_threads.restype = ctypes.c_int32
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def max_threads() -> int:
    return int(_load().kbo_max_threads())


def prune(seg_off, flops, bytes_, peak_flops, peak_bw, incumbent):
    lib = _load()
    seg_off = _c(seg_off, np.int32)
    G = len(seg_off) - 1
    N = int(seg_off[-1])
    flops = _c(flops, np.float32)
    bytes_ = _c(bytes_, np.float32)
    incumbent = _c(incumbent, np.float32)
    bound = np.empty(N, dtype=np.float32)
    alive = np.empty(N, dtype=np.uint8)
    lib.kbo_prune(ctypes.c_int32(G), _p(seg_off), _p(flops), _p(bytes_),
                  ctypes.c_float(peak_flops), ctypes.c_float(peak_bw),
                  _p(incumbent), _p(bound), _p(alive))
    return bound, alive


def assign(seg_off, koff, X, cent):
    lib = _load()
    seg_off = _c(seg_off, np.int32)
    koff = _c(koff, np.int32)
    X = _c(X, np.float32)
    cent = _c(cent, np.float32)
    G = len(seg_off) - 1
    N, D = X.shape
    a = np.empty(N, dtype=np.int32)
    mind2 = np.empty(N, dtype=np.float64)
    flag = np.empty(N, dtype=np.uint8)
    lib.kbo_assign(ctypes.c_int32(G), ctypes.c_int32(D), _p(seg_off), _p(koff),
                   _p(X), _p(cent), _p(a), _p(mind2), _p(flag))
    return a, mind2, flag


def update(seg_off, koff, X, cent_in, assign_):
    lib = _load()
    seg_off = _c(seg_off, np.int32)
    koff = _c(koff, np.int32)
    X = _c(X, np.float32)
    cent_in = _c(cent_in, np.float32)
    assign_ = _c(assign_, np.int32)
    G = len(seg_off) - 1
    N, D = X.shape
    Ksum = int(koff[-1])
    cent_out = np.empty((Ksum, D), dtype=np.float32)
    counts = np.empty(Ksum, dtype=np.int32)
    lib.kbo_update(ctypes.c_int32(G), ctypes.c_int32(D), _p(seg_off), _p(koff),
                   _p(X), _p(cent_in), _p(assign_), _p(cent_out), _p(counts))
    return cent_out, counts


def objective(seg_off, mind2):
    lib = _load()
    seg_off = _c(seg_off, np.int32)
    mind2 = _c(mind2, np.float64)
    G = len(seg_off) - 1
    J = np.empty(G, dtype=np.float64)
    lib.kbo_objective(ctypes.c_int32(G), _p(seg_off), _p(mind2), _p(J))
    return J


def cluster_step(seg_off, koff, X, cent_in):
    """One Lloyd step.  Returns a namespace with assign, cent, counts,
    objective (fp64), flag (near-tie per candidate) and mind2."""
    lib = _load()
    seg_off = _c(seg_off, np.int32)
    koff = _c(koff, np.int32)
    X = _c(X, np.float32)
    cent_in = _c(cent_in, np.float32)
    G = len(seg_off) - 1
    N, D = X.shape
    Ksum = int(koff[-1])
    a = np.empty(N, dtype=np.int32)
    cent_out = np.empty((Ksum, D), dtype=np.float32)
    counts = np.empty(Ksum, dtype=np.int32)
    J = np.empty(G, dtype=np.float64)
    mind2 = np.empty(N, dtype=np.float64)
    flag = np.empty(N, dtype=np.uint8)
    lib.kbo_cluster_step(ctypes.c_int32(G), ctypes.c_int32(D), _p(seg_off),
                         _p(koff), _p(X), _p(cent_in), _p(a), _p(cent_out),
                         _p(counts), _p(J), _p(mind2), _p(flag))
    return SimpleNamespace(assign=a, cent=cent_out, counts=counts, objective=J,
                           flag=flag, mind2=mind2)


def cluster(seg_off, koff, X, iters, cent_init=None):
    """iters Lloyd steps from cent_init (default: first K_g rows)."""
    lib = _load()
    seg_off = _c(seg_off, np.int32)
    koff = _c(koff, np.int32)
    X = _c(X, np.float32)
    if cent_init is not None:
        cent_init = _c(cent_init, np.float32)
    G = len(seg_off) - 1
    N, D = X.shape
    Ksum = int(koff[-1])
    a = np.full(N, -1, dtype=np.int32)
    cent = np.empty((Ksum, D), dtype=np.float32)
    counts = np.full(Ksum, -1, dtype=np.int32)
    J = np.full(G, np.nan, dtype=np.float64)
    dirty = np.zeros(G, dtype=np.uint8)
    lib.kbo_cluster(ctypes.c_int32(G), ctypes.c_int32(D), _p(seg_off), _p(koff),
                    _p(X), _p(cent_init), ctypes.c_int32(iters), _p(a), _p(cent),
                    _p(counts), _p(J), _p(dirty))
    return SimpleNamespace(assign=a, cent=cent, counts=counts, objective=J,
                           dirty=dirty)


def ucb_select(seg_off, koff, S, assign_, alive, bound, visits, rsum, t, c,
               prior_n=0.0, prior_mu=0.5, M=None):
    lib = _load()
    seg_off = _c(seg_off, np.int32)
    koff = _c(koff, np.int32)
    assign_ = _c(assign_, np.int32)
    alive = None if alive is None else _c(alive, np.uint8)
    bound = None if bound is None else _c(bound, np.float32)
    M = None if M is None else _c(M, np.uint8)
    visits = _c(visits, np.int32)
    rsum = _c(rsum, np.float32)
    t = _c(t, np.int64)
    G = len(seg_off) - 1
    Ksum = int(koff[-1])
    Ncs = np.empty((Ksum, S), dtype=np.int64)
    mu = np.empty((Ksum, S), dtype=np.float64)
    ucb = np.empty((Ksum, S), dtype=np.float64)
    sel = np.empty((G, 3), dtype=np.int32)
    near = np.empty(G, dtype=np.uint8)
    lib.kbo_ucb_select(ctypes.c_int32(G), ctypes.c_int32(S), _p(seg_off), _p(koff),
                       _p(assign_), _p(alive), _p(bound), _p(visits), _p(rsum),
                       _p(t), ctypes.c_double(c), ctypes.c_double(prior_n),
                       ctypes.c_double(prior_mu), _p(M), _p(Ncs), _p(mu), _p(ucb),
                       _p(sel), _p(near))
    return SimpleNamespace(Ncs=Ncs, mu=mu, ucb=ucb, sel=sel, near=near)


def philox4x32_10(ctr, key):
    lib = _load()
    c = (ctypes.c_uint32 * 4)(*[int(v) for v in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(v) for v in key])
    out = (ctypes.c_uint32 * 4)()
    lib.kbo_philox4x32_10(c, k, out)
    return [int(v) for v in out]


def uniform(seed, draw, k):
    lib = _load()
    lib.kbo_uniform.restype = ctypes.c_double
    return float(lib.kbo_uniform(ctypes.c_uint64(seed), ctypes.c_uint64(draw), ctypes.c_int32(k)))


def sample(seg_off, assign_, alive, bound, incumbent, sel, seed, draw, tau=1.0):
    """Draw k_t in the chosen cluster of every search.  Returns a namespace with
    ksel (global candidate index or -1) and near (near-tie of the two best keys)."""
    lib = _load()
    seg_off = _c(seg_off, np.int32)
    assign_ = _c(assign_, np.int32)
    if alive is not None:
        alive = _c(alive, np.uint8)
    bound = _c(bound, np.float32)
    incumbent = _c(incumbent, np.float32)
    sel = _c(sel, np.int32)
    G = len(seg_off) - 1
    ksel = np.empty(G, dtype=np.int32)
    near = np.empty(G, dtype=np.uint8)
    lib.kbo_sample(ctypes.c_int32(G), _p(seg_off), _p(assign_), _p(alive), _p(bound),
                   _p(incumbent), _p(sel), ctypes.c_uint64(seed), ctypes.c_uint64(draw),
                   ctypes.c_double(tau), _p(ksel), _p(near))
    return SimpleNamespace(ksel=ksel, near=near)


def cluster_geometry(seg_off, koff, X, cent, assign_):
    """Representative (member nearest the centroid) and radius of every cluster,
    and the squared distance of every candidate to its centroid."""
    lib = _load()
    seg_off = _c(seg_off, np.int32)
    koff = _c(koff, np.int32)
    X = _c(X, np.float32)
    cent = _c(cent, np.float32)
    assign_ = _c(assign_, np.int32)
    G = len(seg_off) - 1
    N, D = X.shape
    Ksum = int(koff[-1])
    rep = np.full(Ksum, -1, dtype=np.int32)
    radius = np.zeros(Ksum, dtype=np.float64)
    dist2 = np.zeros(N, dtype=np.float64)
    lib.kbo_cluster_geometry(ctypes.c_int32(G), ctypes.c_int32(D), _p(seg_off), _p(koff),
                             _p(X), _p(cent), _p(assign_), _p(rep), _p(radius), _p(dist2))
    return SimpleNamespace(rep=rep, radius=radius, dist2=dist2)


def cluster_diameter(seg_off, koff, X, assign_):
    """diam(C_i) of every cluster: largest member-to-member distance (fp64)."""
    lib = _load()
    seg_off = _c(seg_off, np.int32)
    koff = _c(koff, np.int32)
    X = _c(X, np.float32)
    assign_ = _c(assign_, np.int32)
    G = len(seg_off) - 1
    N, D = X.shape
    diam = np.zeros(int(koff[-1]), dtype=np.float64)
    lib.kbo_cluster_diameter(ctypes.c_int32(G), ctypes.c_int32(D), _p(seg_off), _p(koff), _p(X),
                             _p(assign_), _p(diam))
    return diam


def seed_farthest(seg_off, koff, X):
    """Farthest-point initial centroids.  Returns cent [Ksum, D] and pick [Ksum]
    (global candidate index of every chosen row)."""
    lib = _load()
    seg_off = _c(seg_off, np.int32)
    koff = _c(koff, np.int32)
    X = _c(X, np.float32)
    G = len(seg_off) - 1
    N, D = X.shape
    Ksum = int(koff[-1])
    cent = np.zeros((Ksum, D), dtype=np.float32)
    pick = np.full(Ksum, -1, dtype=np.int32)
    lib.kbo_seed_farthest(ctypes.c_int32(G), ctypes.c_int32(D), _p(seg_off), _p(koff), _p(X),
                          _p(cent), _p(pick))
    return SimpleNamespace(cent=cent, pick=pick)


def seed_dsquared(seg_off, koff, X, seed, draw0):
    """k-means++-style initial centroids (D^2-weighted draws).  Returns cent, pick
    and near (per search: some draw had its two best keys within 1e-6 relative)."""
    lib = _load()
    seg_off = _c(seg_off, np.int32)
    koff = _c(koff, np.int32)
    X = _c(X, np.float32)
    G = len(seg_off) - 1
    N, D = X.shape
    Ksum = int(koff[-1])
    cent = np.zeros((Ksum, D), dtype=np.float32)
    pick = np.full(Ksum, -1, dtype=np.int32)
    near = np.zeros(G, dtype=np.uint8)
    lib.kbo_seed_dsquared(ctypes.c_int32(G), ctypes.c_int32(D), _p(seg_off), _p(koff), _p(X),
                          ctypes.c_uint64(seed), ctypes.c_uint64(draw0), _p(cent), _p(pick),
                          _p(near))
    return SimpleNamespace(cent=cent, pick=pick, near=near)


def strategy_mask(koff, S, h, target, rep, theta_sat):
    lib = _load()
    koff = _c(koff, np.int32)
    h = _c(h, np.float32)
    target = _c(target, np.int32)
    rep = _c(rep, np.int32)
    G = len(koff) - 1
    Ksum = int(koff[-1])
    R = h.shape[1]
    M = np.zeros((Ksum, S), dtype=np.uint8)
    nvalid = np.zeros(G, dtype=np.int32)
    lib.kbo_strategy_mask(ctypes.c_int32(G), ctypes.c_int32(S), ctypes.c_int32(R), _p(koff),
                          _p(h), _p(target), _p(rep), ctypes.c_float(theta_sat), _p(M),
                          _p(nvalid))
    return SimpleNamespace(M=M, nvalid=nvalid)


def sample_signature(seg_off, assign_, alive, h, target, theta_sat, sel, seed, draw, tau=1.0):
    lib = _load()
    seg_off = _c(seg_off, np.int32)
    assign_ = _c(assign_, np.int32)
    if alive is not None:
        alive = _c(alive, np.uint8)
    h = _c(h, np.float32)
    target = _c(target, np.int32)
    sel = _c(sel, np.int32)
    G = len(seg_off) - 1
    ksel = np.empty(G, dtype=np.int32)
    near = np.empty(G, dtype=np.uint8)
    lib.kbo_sample_signature(ctypes.c_int32(G), ctypes.c_int32(h.shape[1]), _p(seg_off),
                             _p(assign_), _p(alive), _p(h), _p(target),
                             ctypes.c_float(theta_sat), _p(sel), ctypes.c_uint64(seed),
                             ctypes.c_uint64(draw), ctypes.c_double(tau), _p(ksel), _p(near))
    return SimpleNamespace(ksel=ksel, near=near)


def update_stats(koff, S, sel, ksel, reward, ok, prior_n, visits, rsum, Ncs, mu, t):
    """Applies the end-of-iteration update; returns updated COPIES of visits,
    rsum, Ncs (int32), mu (fp32) and t."""
    lib = _load()
    koff = _c(koff, np.int32)
    sel = _c(sel, np.int32)
    ksel = _c(ksel, np.int32)
    reward = _c(reward, np.float32)
    ok = _c(ok, np.uint8)
    visits = np.array(visits, dtype=np.int32, order="C", copy=True)
    rsum = np.array(rsum, dtype=np.float32, order="C", copy=True)
    Ncs = np.array(Ncs, dtype=np.int32, order="C", copy=True)
    mu = np.array(mu, dtype=np.float32, order="C", copy=True)
    t = np.array(t, dtype=np.int64, order="C", copy=True)
    G = len(koff) - 1
    lib.kbo_update_stats(ctypes.c_int32(G), ctypes.c_int32(S), _p(koff), _p(sel), _p(ksel),
                         _p(reward), _p(ok), ctypes.c_double(prior_n), _p(visits), _p(rsum),
                         _p(Ncs), _p(mu), _p(t))
    return SimpleNamespace(visits=visits, rsum=rsum, Ncs=Ncs, mu=mu, t=t)


def round_(b, iters=None):
    """Full round on a synth.Batch-like object (duck-typed: only attributes are
    read)."""
    lib = _load()
    iters = b.iters if iters is None else iters
    seg_off = _c(b.seg_off, np.int32)
    koff = _c(b.koff, np.int32)
    X = _c(b.X, np.float32)
    G = len(seg_off) - 1
    N, D = X.shape
    S = int(b.S)
    Ksum = int(koff[-1])
    flops = _c(b.flops, np.float32)
    bytes_ = _c(b.bytes_, np.float32)
    inc = _c(b.incumbent, np.float32)
    visits = _c(b.visits, np.int32)
    rsum = _c(b.rsum, np.float32)
    t = _c(b.t, np.int64)
    out = SimpleNamespace(
        bound=np.empty(N, dtype=np.float32), alive=np.empty(N, dtype=np.uint8),
        assign=np.full(N, -1, dtype=np.int32),
        cent=np.empty((Ksum, D), dtype=np.float32),
        counts=np.full(Ksum, -1, dtype=np.int32),
        objective=np.full(G, np.nan, dtype=np.float64),
        Ncs=np.empty((Ksum, S), dtype=np.int64),
        mu=np.empty((Ksum, S), dtype=np.float64),
        ucb=np.empty((Ksum, S), dtype=np.float64),
        sel=np.empty((G, 3), dtype=np.int32),
        dirty=np.zeros(G, dtype=np.uint8), near=np.zeros(G, dtype=np.uint8))
    lib.kbo_round(ctypes.c_int32(G), ctypes.c_int32(D), ctypes.c_int32(S),
                  _p(seg_off), _p(koff), _p(X), _p(flops), _p(bytes_), _p(inc),
                  _p(visits), _p(rsum), _p(t), ctypes.c_float(b.peak_flops),
                  ctypes.c_float(b.peak_bw), ctypes.c_double(b.c),
                  ctypes.c_double(b.prior_n), ctypes.c_double(b.prior_mu),
                  ctypes.c_int32(iters), _p(out.bound), _p(out.alive),
                  _p(out.assign), _p(out.cent), _p(out.counts), _p(out.objective),
                  _p(out.Ncs), _p(out.mu), _p(out.ucb), _p(out.sel), _p(out.dirty),
                  _p(out.near))
    return out


def iterate(seg_off, koff, S, X, h, target, theta_sat, alive, reward, ok, visits, rsum, t,
            assign_, cent, counts, objective, rep, M, rounds, tau_recluster, t0, warm_start,
            iters, c, prior_n, prior_mu, seed, draw0, temperature=1.0):
    """Several iterations of Alg. 1 composed from the functions above, in the
    order the algorithm states them.  Round r, iteration number it = t0 + r:
      if tau_recluster > 0 and it % tau_recluster == 0: K-Means (`iters` Lloyd steps,
        from the first K_g rows or, warm_start, from the current centroids) on
        every search with N_g >= 2 K_g - the others keep their clustering - then the
        representatives k_c and the mask of Eq. 5 from their signatures;
      cluster-arm statistics re-aggregated from the per-candidate history, masked
        UCB argmax (Eq. 6); draw of k_t with theta_sat - h; statistics update.
    Returns the per-round logs (sel, ksel and the union of the near-tie flags that
    make a search's later rounds incomparable) and the final state."""
    seg_off = _c(seg_off, np.int32)
    koff = _c(koff, np.int32)
    G = len(seg_off) - 1
    visits = np.array(visits, dtype=np.int32, copy=True)
    rsum = np.array(rsum, dtype=np.float32, copy=True)
    t = np.array(t, dtype=np.int64, copy=True)
    assign_ = np.array(assign_, dtype=np.int32, copy=True)
    cent = np.array(cent, dtype=np.float32, copy=True)
    counts = np.array(counts, dtype=np.int32, copy=True)
    objective = np.array(objective, dtype=np.float64, copy=True)
    rep = np.array(rep, dtype=np.int32, copy=True)
    M = np.array(M, dtype=np.uint8, copy=True)
    ng = np.diff(seg_off)
    kg = np.diff(koff)
    sel_log = np.zeros((rounds, G, 3), np.int32)
    ksel_log = np.zeros((rounds, G), np.int32)
    doubt = np.zeros((rounds, G), np.uint8)     # a near-tie seen in this round (any stage)
    Ncs = mu = ucb = None
    for r in range(rounds):
        it = t0 + r
        if tau_recluster > 0 and it % tau_recluster == 0:
            cl = cluster(seg_off, koff, X, iters, cent_init=cent if warm_start else None)
            go = (ng >= 2 * kg) & (ng > 0)
            gp = np.repeat(go, ng)
            gk = np.repeat(go, kg)
            assign_[gp] = cl.assign[gp]
            cent[gk] = cl.cent[gk]
            counts[gk] = cl.counts[gk]
            objective[go] = cl.objective[go]
            doubt[r] |= (cl.dirty != 0) & go
            geo = cluster_geometry(seg_off, koff, X, cent, assign_)
            rep = geo.rep
            M = strategy_mask(koff, S, h, target, rep, theta_sat).M
        u = ucb_select(seg_off, koff, S, assign_, alive, None, visits, rsum, t, c, prior_n,
                       prior_mu, M=M)
        s = sample_signature(seg_off, assign_, alive, h, target, theta_sat, u.sel, seed, draw0 + r,
                             temperature)
        doubt[r] |= (u.near != 0) | (s.near != 0)
        sel_log[r] = u.sel
        ksel_log[r] = s.ksel
        up = update_stats(koff, S, u.sel, s.ksel, reward[r], ok[r], prior_n, visits, rsum,
                          u.Ncs.astype(np.int32), u.mu.astype(np.float32), t)
        visits, rsum, t = up.visits, up.rsum, up.t
        Ncs, mu, ucb = up.Ncs, up.mu, u.ucb
    return SimpleNamespace(sel_log=sel_log, ksel_log=ksel_log, doubt=doubt, visits=visits,
                           rsum=rsum, t=t, assign=assign_, cent=cent, counts=counts,
                           objective=objective, rep=rep, M=M, Ncs=Ncs, mu=mu, ucb=ucb)
