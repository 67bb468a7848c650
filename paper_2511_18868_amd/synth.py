"""Seeded synthetic inputs for the arm-scoring pass (prune -> cluster -> UCB select).

This module only draws inputs.  It holds none of the method's arithmetic: no
distance, no centroid update, no UCB score.  Both the CPU oracle's tests and the
GPU path's tests/benchmarks read their inputs from here, so the two see the
same bytes.

The synthetic traces stand in for the behavioural feature vectors phi(k)
(Sec. 3.2, Eq. 4) and hardware signatures that profiling real kernels would
give: a handful of behaviour clusters per search, heavy-tailed counters,
rewards in [0, 1] (Sec. 2.2) and small integer visit counts (Alg. 1).

One documented exception to "no arithmetic": the incumbent runtime of a search
is *defined* as the lower median of that search's per-candidate roofline
runtimes max(flops/peak_flops, bytes/peak_bw), so the generator has to evaluate
that expression (numpy, fp32) to draw the input.  Neither the oracle nor the GPU
path calls this code.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

BASE_SEED = 20251118
PEAK_FLOPS = 2.5e15   # dense bf16 MFMA peak of the target GPU, flop/s
PEAK_BW = 8.0e12      # HBM3E peak, B/s


@dataclass
class Batch:
    """One batch of G independent searches stored as contiguous segments."""
    name: str
    G: int
    D: int
    S: int
    iters: int
    seg_off: np.ndarray      # [G+1] int32
    koff: np.ndarray         # [G+1] int32
    X: np.ndarray            # [N, D] float32, row-major
    flops: np.ndarray        # [N] float32
    bytes_: np.ndarray       # [N] float32
    incumbent: np.ndarray    # [G] float32
    visits: np.ndarray       # [N, S] int32
    rsum: np.ndarray         # [N, S] float32
    t: np.ndarray            # [G] int64
    peak_flops: float = PEAK_FLOPS
    peak_bw: float = PEAK_BW
    c: float = float(np.float32(math.sqrt(2.0)))
    prior_n: float = 0.0
    prior_mu: float = 0.5
    extra: Dict = field(default_factory=dict)

    @property
    def N(self) -> int:
        return int(self.seg_off[-1])

    @property
    def Ksum(self) -> int:
        return int(self.koff[-1])

    @property
    def Kmax(self) -> int:
        return int(np.max(np.diff(self.koff))) if self.G else 0

    @property
    def Nmax(self) -> int:
        return int(np.max(np.diff(self.seg_off))) if self.G else 0


def concat(a: Batch, b: Batch, name: str = "concat") -> Batch:
    """The searches of `a` followed by those of `b` as one batch (same D and S)."""
    assert a.D == b.D and a.S == b.S
    cat = np.concatenate
    return Batch(name=name, G=a.G + b.G, D=a.D, S=a.S, iters=a.iters,
                 seg_off=cat([a.seg_off, a.seg_off[-1] + b.seg_off[1:]]).astype(np.int32),
                 koff=cat([a.koff, a.koff[-1] + b.koff[1:]]).astype(np.int32),
                 X=cat([a.X, b.X]), flops=cat([a.flops, b.flops]), bytes_=cat([a.bytes_, b.bytes_]),
                 incumbent=cat([a.incumbent, b.incumbent]), visits=cat([a.visits, b.visits]),
                 rsum=cat([a.rsum, b.rsum]), t=cat([a.t, b.t]), peak_flops=a.peak_flops,
                 peak_bw=a.peak_bw, c=a.c, prior_n=a.prior_n, prior_mu=a.prior_mu)


def _zscore(a: np.ndarray) -> np.ndarray:
    """Per-feature z-score over the rows, population std, zero variance -> 0."""
    mu = a.mean(axis=0)
    sd = a.std(axis=0)
    out = a - mu
    nz = sd > 0
    out[:, nz] /= sd[nz]
    out[:, ~nz] = 0.0
    return out


def _features_lognormal(rng, n, d, ncentres):
    # config 1: log-normal counters (sigma = 1) around seeded Gaussian centres
    centres = rng.standard_normal((ncentres, d))
    lab = rng.integers(0, ncentres, size=n)
    raw = np.exp(centres[lab] + rng.standard_normal((n, d)))
    return _zscore(raw)


def _features_gauss(rng, n, d, ncentres, spread=3.0, sigma=None, weights=None,
                    outlier_frac=0.0):
    centres = spread * rng.standard_normal((ncentres, d))
    if weights is None:
        lab = rng.integers(0, ncentres, size=n)
    else:
        lab = rng.choice(ncentres, size=n, p=weights)
    noise = rng.standard_normal((n, d))
    if sigma is not None:
        noise *= sigma[lab][:, None]
    x = centres[lab] + noise
    if outlier_frac > 0.0:
        n_out = int(round(outlier_frac * n))
        lo = x[n_out:].min(axis=0)
        hi = x[n_out:].max(axis=0)
        x[:n_out] = lo + (hi - lo) * rng.random((n_out, d))
    x = x[rng.permutation(n)]
    return _zscore(x)


def _roofline_inputs(rng, seg_off, peak_flops, peak_bw):
    n = int(seg_off[-1])
    flops = (10.0 ** rng.uniform(6.0, 12.0, size=n)).astype(np.float32)
    bytes_ = (10.0 ** rng.uniform(6.0, 12.0, size=n)).astype(np.float32)
    # incumbent = lower median of the search's fp32 roofline runtimes (input
    # definition; see the module docstring)
    rt = np.maximum(flops / np.float32(peak_flops), bytes_ / np.float32(peak_bw))
    G = len(seg_off) - 1
    inc = np.zeros(G, dtype=np.float32)
    for g in range(G):
        a, b = int(seg_off[g]), int(seg_off[g + 1])
        if b > a:
            m = (b - a - 1) // 2
            inc[g] = np.partition(rt[a:b], m)[m]
        else:
            inc[g] = np.float32(np.inf)
    return flops, bytes_, inc


def _ucb_inputs(rng, seg_off, S):
    n = int(seg_off[-1])
    G = len(seg_off) - 1
    visits = np.empty((n, S), dtype=np.int32)
    rsum = np.empty((n, S), dtype=np.float32)
    # chunked so the fp64/int64 temporaries of the large configs stay small
    step = max(1, (1 << 22) // max(S, 1))
    for a in range(0, n, step):
        b = min(n, a + step)
        v = rng.poisson(5.0, size=(b - a, S)) + 1
        p = rng.random((b - a, S))
        visits[a:b] = v
        rsum[a:b] = rng.binomial(v, p)
    t = np.zeros(G, dtype=np.int64)
    if n:
        rowsum = visits.sum(axis=1, dtype=np.int64)
        cs = np.concatenate([[0], np.cumsum(rowsum)])
        t = (cs[seg_off[1:]] - cs[seg_off[:-1]]).astype(np.int64)
    t = np.maximum(t, 1)
    return visits, rsum, t


def _finish(name, rng, seg_off, koff, X, D, S, iters, extra=None) -> Batch:
    seg_off = np.asarray(seg_off, dtype=np.int32)
    koff = np.asarray(koff, dtype=np.int32)
    r_prune, r_ucb = rng.spawn(2)
    flops, bytes_, inc = _roofline_inputs(r_prune, seg_off, PEAK_FLOPS, PEAK_BW)
    visits, rsum, t = _ucb_inputs(r_ucb, seg_off, S)
    return Batch(name=name, G=len(seg_off) - 1, D=D, S=S, iters=iters,
                 seg_off=seg_off, koff=koff,
                 X=np.ascontiguousarray(X, dtype=np.float32),
                 flops=flops, bytes_=bytes_, incumbent=inc,
                 visits=visits, rsum=rsum, t=t, extra=extra or {})


def config1(seed: Optional[int] = None, N=256, D=16, K=8, S=8, iters=20) -> Batch:
    rng = np.random.default_rng(BASE_SEED + 1 if seed is None else seed)
    X = _features_lognormal(rng, N, D, 8)
    return _finish("config1", rng, [0, N], [0, K], X, D, S, iters)


def config2(seed: Optional[int] = None, N=4096, D=32, K=32, S=16, iters=30) -> Batch:
    rng = np.random.default_rng(BASE_SEED + 2 if seed is None else seed)
    X = _features_gauss(rng, N, D, 32)
    return _finish("config2", rng, [0, N], [0, K], X, D, S, iters)


def config3(seed: Optional[int] = None, G=1024, Ng=512, D=32, K=16, S=16, iters=25) -> Batch:
    rng = np.random.default_rng(BASE_SEED + 3 if seed is None else seed)
    subs = rng.spawn(G)
    X = np.empty((G * Ng, D), dtype=np.float32)
    for g in range(G):
        X[g * Ng:(g + 1) * Ng] = _features_gauss(subs[g], Ng, D, 16)
    seg_off = np.arange(G + 1, dtype=np.int64) * Ng
    koff = np.arange(G + 1, dtype=np.int64) * K
    return _finish("config3", rng, seg_off, koff, X, D, S, iters)


def config4(seed: Optional[int] = None, N=1 << 20, D=64, K=256, S=4, iters=10,
            ncentres=256) -> Batch:
    rng = np.random.default_rng(BASE_SEED + 4 if seed is None else seed)
    X = _features_gauss(rng, N, D, ncentres, outlier_frac=0.10)
    return _finish("config4", rng, [0, N], [0, K], X, D, S, iters)


def config5(seed: Optional[int] = None, G=4096, nmin=64, nmax=4096, D=48, S=32,
            iters=20, kcap=64, kdiv=16) -> Batch:
    rng = np.random.default_rng(BASE_SEED + 5 if seed is None else seed)
    ng = np.rint(np.exp(rng.uniform(math.log(nmin), math.log(nmax), size=G)))
    ng = np.clip(ng, nmin, nmax).astype(np.int64)
    kg = np.minimum(kcap, ng // kdiv).astype(np.int64)
    kg = np.maximum(kg, 1)
    seg_off = np.concatenate([[0], np.cumsum(ng)])
    koff = np.concatenate([[0], np.cumsum(kg)])
    subs = rng.spawn(G)
    X = np.empty((int(seg_off[-1]), D), dtype=np.float32)
    for g in range(G):
        r = subs[g]
        k = int(kg[g])
        sigma = r.uniform(0.5, 1.5, size=k)
        w = r.dirichlet(np.ones(k))
        X[seg_off[g]:seg_off[g + 1]] = _features_gauss(
            r, int(ng[g]), D, k, sigma=sigma, weights=w)
    return _finish("config5", rng, seg_off, koff, X, D, S, iters)


def paper_scale(seed: int = 11, G=183) -> Batch:
    """A batch at the scale the paper itself runs (Sec. 3.6 and its experimental
    setup: 183 benchmark kernels, one search each, a frontier that grows by one kernel
    per iteration up to T = 40, K = 3 clusters, |S| = 6 strategies, a handful of
    profiler features)."""
    b = config5(seed=seed, G=G, nmin=12, nmax=41, D=5, S=6, iters=10, kcap=3, kdiv=4)
    b.name = "paper_scale"
    return b


def paper_shape(seed: int = 7, N=21, D=5, K=3, S=6, iters=10) -> Batch:
    """A search with the sizes the paper itself runs (Sec. 3.6: K = 3, |S| = 6,
    5 features, a frontier of at most T + 1 = 21 kernels) and its constants
    (c = 2.0, initial statistics N = 1, mu = 0.5 from Alg. 1)."""
    rng = np.random.default_rng(seed)
    X = _features_gauss(rng, N, D, K)
    b = _finish("paper_shape", rng, [0, N], [0, K], X, D, S, iters)
    b.c = 2.0
    b.prior_n = 1.0
    b.prior_mu = 0.5
    return b


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


def make(config: int, **kw) -> Batch:
    return CONFIGS[config](**kw)


def random_centroids(batch: Batch, seed: int = 0) -> np.ndarray:
    """cent_in for a single-step test: for each search, K_g distinct rows of it
    picked at random (fp32, [Ksum, D])."""
    rng = np.random.default_rng(seed)
    out = np.empty((batch.Ksum, batch.D), dtype=np.float32)
    for g in range(batch.G):
        a, b = int(batch.seg_off[g]), int(batch.seg_off[g + 1])
        k0, k1 = int(batch.koff[g]), int(batch.koff[g + 1])
        if k1 > k0:
            rows = rng.choice(b - a, size=k1 - k0, replace=False)
            out[k0:k1] = batch.X[a + rows]
    return out


def signatures(batch: Batch, R: int = 3, seed: int = 0):
    """Hardware signatures for the paper's own form of the mask (Sec. 3.2): for
    every candidate the share of peak throughput of R resources (the paper uses
    DRAM, L2 and SM), drawn from a Beta(2, 2) so that a 75 % threshold cuts off a
    sizeable minority, a few of them set exactly to the threshold; and the resource
    each strategy targets, round-robin over the resources.  Returns (h [N,R] fp32,
    target [S] int32, theta_sat)."""
    rng = np.random.default_rng(BASE_SEED + 1000 + seed)
    h = rng.beta(2.0, 2.0, size=(batch.N, R)).astype(np.float32)
    theta = float(np.float32(0.75))
    exact = rng.random((batch.N, R)) < 0.02
    h[exact] = np.float32(theta)
    target = (np.arange(batch.S) % R).astype(np.int32)
    return h, target, theta


def feedback(batch: Batch, seed: int = 0):
    """Outcome of one generation step per search: a reward in [0, 1] (Sec. 2.2) and
    whether the generated kernel passed verification (about four in five do)."""
    rng = np.random.default_rng(BASE_SEED + 2000 + seed)
    reward = rng.uniform(0.0, 1.0, batch.G).astype(np.float32)
    ok = (rng.random(batch.G) < 0.8).astype(np.uint8)
    reward[ok == 0] = 0.0
    return reward, ok
