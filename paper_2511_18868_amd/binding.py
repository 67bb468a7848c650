"""Thin ctypes binding of libkernelband.so: same names as include/kb.h,
argument marshalling only.  torch supplies device memory and the stream; every
step of the path runs in the library's HIP kernels.  There is no CPU fallback:
a missing library raises."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkernelband.so")

KB_OK, KB_EINVAL, KB_EUNSUPPORTED, KB_EWORKSPACE, KB_EDEVICE = range(5)


class KBError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().kb_status_str(status).decode()
        super().__init__(f"{where}: {msg}")


class kb_batch(ctypes.Structure):
    _fields_ = [("G", ctypes.c_int32), ("D", ctypes.c_int32), ("S", ctypes.c_int32),
                ("N", ctypes.c_int64), ("Kmax", ctypes.c_int32), ("Ksum", ctypes.c_int32),
                ("Nmax", ctypes.c_int32), ("seg_off", ctypes.c_void_p),
                ("koff", ctypes.c_void_p)]


class kb_params(ctypes.Structure):
    _fields_ = [("peak_flops", ctypes.c_float), ("peak_bw", ctypes.c_float),
                ("c", ctypes.c_float), ("prior_n", ctypes.c_float),
                ("prior_mu", ctypes.c_float), ("iters", ctypes.c_int32),
                ("scorer", ctypes.c_int32), ("stop_early", ctypes.c_int32)]


class kb_round_io(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in (
        "X", "flops", "bytes", "incumbent", "visits", "rsum", "t", "bound", "alive",
        "assign", "cent", "counts", "objective", "Ncs", "mu", "ucb", "sel")]


class kb_sample_params(ctypes.Structure):
    _fields_ = [("seed", ctypes.c_uint64), ("draw", ctypes.c_uint64), ("tau", ctypes.c_float)]


class kb_iterate_params(ctypes.Structure):
    _fields_ = [("rounds", ctypes.c_int32), ("tau_recluster", ctypes.c_int32),
                ("t0", ctypes.c_int64), ("warm_start", ctypes.c_int32), ("R", ctypes.c_int32),
                ("theta_sat", ctypes.c_float), ("sample", kb_sample_params)]


class kb_iterate_io(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in (
        "X", "h", "target", "alive", "reward", "ok", "visits", "rsum", "t", "assign", "cent",
        "counts", "objective", "rep", "radius", "M", "nvalid", "Ncs", "mu", "ucb", "sel_log",
        "ksel_log")]


_lib = None


def lib() -> ctypes.CDLL:
    """Load libkernelband.so (built by paper_2511_18868_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with "
                "`python -m paper_2511_18868_amd.build` (there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        pb, pp = ctypes.POINTER(kb_batch), ctypes.POINTER(kb_params)
        L.kb_workspace_bytes.restype = sz
        L.kb_workspace_bytes.argtypes = [pb, pp]
        L.kb_prune.restype = ctypes.c_int
        L.kb_prune.argtypes = [pb, pp, vp, vp, vp, vp, vp, vp]
        L.kb_cluster_step.restype = ctypes.c_int
        L.kb_cluster_step.argtypes = [pb, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.kb_cluster.restype = ctypes.c_int
        L.kb_cluster.argtypes = [pb, pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.kb_ucb_select.restype = ctypes.c_int
        L.kb_ucb_select.argtypes = [pb, pp] + [vp] * 10 + [vp, sz, vp]
        L.kb_ucb_select_static.restype = ctypes.c_int
        L.kb_ucb_select_static.argtypes = [pb, pp] + [vp] * 10 + [vp]
        L.kb_iterate.restype = ctypes.c_int
        L.kb_iterate.argtypes = [pb, pp, ctypes.POINTER(kb_iterate_params),
                                 ctypes.POINTER(kb_iterate_io), vp, sz, vp]
        L.kb_round.restype = ctypes.c_int
        L.kb_round.argtypes = [pb, pp, ctypes.POINTER(kb_round_io), vp, sz, vp]
        L.kb_sample.restype = ctypes.c_int
        L.kb_sample.argtypes = [pb, ctypes.POINTER(kb_sample_params)] + [vp] * 6 + [vp, sz, vp]
        L.kb_sample_signature.restype = ctypes.c_int
        L.kb_sample_signature.argtypes = [pb, ctypes.POINTER(kb_sample_params), vp, vp,
                                          ctypes.c_int32, vp, vp, ctypes.c_float, vp, vp,
                                          vp, sz, vp]
        L.kb_cluster_geometry.restype = ctypes.c_int
        L.kb_cluster_geometry.argtypes = [pb] + [vp] * 5 + [vp, sz, vp]
        L.kb_strategy_mask.restype = ctypes.c_int
        L.kb_strategy_mask.argtypes = [pb, ctypes.c_int32, vp, vp, vp, ctypes.c_float, vp, vp, vp]
        L.kb_ucb_select_masked.restype = ctypes.c_int
        L.kb_ucb_select_masked.argtypes = [pb, pp] + [vp] * 11 + [vp, sz, vp]
        L.kb_update_stats.restype = ctypes.c_int
        L.kb_update_stats.argtypes = [pb, pp] + [vp] * 9 + [vp]
        L.kb_seed_farthest.restype = ctypes.c_int
        L.kb_seed_farthest.argtypes = [pb, vp, vp, vp, vp, sz, vp]
        L.kb_seed_dsquared.restype = ctypes.c_int
        L.kb_seed_dsquared.argtypes = [pb, vp, ctypes.c_uint64, ctypes.c_uint64, vp, vp, vp, sz, vp]
        L.kb_cluster_diameter.restype = ctypes.c_int
        L.kb_cluster_diameter.argtypes = [pb, vp, vp, vp, vp, sz, vp]
        L.kb_status_str.restype = ctypes.c_char_p
        L.kb_status_str.argtypes = [ctypes.c_int]
        L.kb_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor, an int, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status: int, where: str, raise_on_error: bool) -> int:
    if status != KB_OK and raise_on_error:
        raise KBError(status, where)
    return status


def make_batch(G, D, S, N, Kmax, Ksum, Nmax, seg_off, koff) -> kb_batch:
    return kb_batch(G, D, S, N, Kmax, Ksum, Nmax, _ptr(seg_off), _ptr(koff))


KB_SCORER_DEFAULT, KB_SCORER_VECTOR_ALU, KB_SCORER_MATRIX_EVERY = range(3)


def make_params(peak_flops=2.5e15, peak_bw=8e12, c=2.0, prior_n=0.0, prior_mu=0.5,
                iters=1, scorer=KB_SCORER_DEFAULT, stop_early=0) -> kb_params:
    return kb_params(peak_flops, peak_bw, c, prior_n, prior_mu, iters, scorer, stop_early)


def kb_workspace_bytes(batch: kb_batch, params: Optional[kb_params] = None) -> int:
    return int(lib().kb_workspace_bytes(ctypes.byref(batch),
                                        ctypes.byref(params) if params is not None else None))


def kb_prune(batch, params, flops, bytes_, incumbent, bound, alive, stream=None, check=True):
    s = lib().kb_prune(ctypes.byref(batch), ctypes.byref(params), _ptr(flops), _ptr(bytes_),
                       _ptr(incumbent), _ptr(bound), _ptr(alive), _stream(stream))
    return _check(s, "kb_prune", check)


def kb_cluster_step(batch, X, cent_in, assign, cent_out, counts, objective, ws, ws_bytes,
                    stream=None, check=True):
    s = lib().kb_cluster_step(ctypes.byref(batch), _ptr(X), _ptr(cent_in), _ptr(assign),
                              _ptr(cent_out), _ptr(counts), _ptr(objective), _ptr(ws),
                              ws_bytes, _stream(stream))
    return _check(s, "kb_cluster_step", check)


def kb_cluster(batch, params, X, cent_init, assign, cent, counts, objective, ws, ws_bytes,
               stream=None, check=True):
    s = lib().kb_cluster(ctypes.byref(batch), ctypes.byref(params), _ptr(X), _ptr(cent_init),
                         _ptr(assign), _ptr(cent), _ptr(counts), _ptr(objective), _ptr(ws),
                         ws_bytes, _stream(stream))
    return _check(s, "kb_cluster", check)


def kb_ucb_select(batch, params, assign, alive, bound, visits, rsum, t, Ncs, mu, ucb, sel,
                  ws, ws_bytes, stream=None, check=True):
    s = lib().kb_ucb_select(ctypes.byref(batch), ctypes.byref(params), _ptr(assign), _ptr(alive),
                            _ptr(bound), _ptr(visits), _ptr(rsum), _ptr(t), _ptr(Ncs), _ptr(mu),
                            _ptr(ucb), _ptr(sel), _ptr(ws), ws_bytes, _stream(stream))
    return _check(s, "kb_ucb_select", check)


def kb_ucb_select_static(batch, params, assign, alive, bound, visits, rsum, t, Ncs, mu, ucb, sel,
                         stream=None, check=True):
    s = lib().kb_ucb_select_static(ctypes.byref(batch), ctypes.byref(params), _ptr(assign),
                                   _ptr(alive), _ptr(bound), _ptr(visits), _ptr(rsum), _ptr(t),
                                   _ptr(Ncs), _ptr(mu), _ptr(ucb), _ptr(sel), _stream(stream))
    return _check(s, "kb_ucb_select_static", check)


def kb_round(batch, params, io: kb_round_io, ws, ws_bytes, stream=None, check=True):
    s = lib().kb_round(ctypes.byref(batch), ctypes.byref(params), ctypes.byref(io), _ptr(ws),
                       ws_bytes, _stream(stream))
    return _check(s, "kb_round", check)


def kb_iterate(batch, params, ip: kb_iterate_params, io: kb_iterate_io, ws, ws_bytes, stream=None,
               check=True):
    s = lib().kb_iterate(ctypes.byref(batch), ctypes.byref(params), ctypes.byref(ip),
                         ctypes.byref(io), _ptr(ws), ws_bytes, _stream(stream))
    return _check(s, "kb_iterate", check)


def kb_sample(batch, sp: kb_sample_params, assign, alive, bound, incumbent, sel, ksel, ws,
              ws_bytes, stream=None, check=True):
    s = lib().kb_sample(ctypes.byref(batch), ctypes.byref(sp), _ptr(assign), _ptr(alive),
                        _ptr(bound), _ptr(incumbent), _ptr(sel), _ptr(ksel), _ptr(ws), ws_bytes,
                        _stream(stream))
    return _check(s, "kb_sample", check)


def kb_sample_signature(batch, sp: kb_sample_params, assign, alive, R, h, target, theta_sat, sel,
                        ksel, ws, ws_bytes, stream=None, check=True):
    s = lib().kb_sample_signature(ctypes.byref(batch), ctypes.byref(sp), _ptr(assign), _ptr(alive),
                                  R, _ptr(h), _ptr(target), theta_sat, _ptr(sel), _ptr(ksel),
                                  _ptr(ws), ws_bytes, _stream(stream))
    return _check(s, "kb_sample_signature", check)


def kb_cluster_geometry(batch, X, cent, assign, rep, radius, ws, ws_bytes, stream=None, check=True):
    s = lib().kb_cluster_geometry(ctypes.byref(batch), _ptr(X), _ptr(cent), _ptr(assign), _ptr(rep),
                                  _ptr(radius), _ptr(ws), ws_bytes, _stream(stream))
    return _check(s, "kb_cluster_geometry", check)


def kb_strategy_mask(batch, R, h, target, rep, theta_sat, M, nvalid, stream=None, check=True):
    s = lib().kb_strategy_mask(ctypes.byref(batch), R, _ptr(h), _ptr(target), _ptr(rep), theta_sat,
                               _ptr(M), _ptr(nvalid), _stream(stream))
    return _check(s, "kb_strategy_mask", check)


def kb_ucb_select_masked(batch, params, assign, alive, bound, M, visits, rsum, t, Ncs, mu, ucb, sel,
                         ws, ws_bytes, stream=None, check=True):
    s = lib().kb_ucb_select_masked(ctypes.byref(batch), ctypes.byref(params), _ptr(assign),
                                   _ptr(alive), _ptr(bound), _ptr(M), _ptr(visits), _ptr(rsum),
                                   _ptr(t), _ptr(Ncs), _ptr(mu), _ptr(ucb), _ptr(sel), _ptr(ws),
                                   ws_bytes, _stream(stream))
    return _check(s, "kb_ucb_select_masked", check)


def kb_update_stats(batch, params, sel, ksel, reward, ok, visits, rsum, Ncs, mu, t, stream=None,
                    check=True):
    s = lib().kb_update_stats(ctypes.byref(batch), ctypes.byref(params), _ptr(sel), _ptr(ksel),
                              _ptr(reward), _ptr(ok), _ptr(visits), _ptr(rsum), _ptr(Ncs), _ptr(mu),
                              _ptr(t), _stream(stream))
    return _check(s, "kb_update_stats", check)


def kb_seed_farthest(batch, X, cent, pick, ws, ws_bytes, stream=None, check=True):
    s = lib().kb_seed_farthest(ctypes.byref(batch), _ptr(X), _ptr(cent), _ptr(pick), _ptr(ws),
                               ws_bytes, _stream(stream))
    return _check(s, "kb_seed_farthest", check)


def kb_seed_dsquared(batch, X, seed, draw0, cent, pick, ws, ws_bytes, stream=None, check=True):
    s = lib().kb_seed_dsquared(ctypes.byref(batch), _ptr(X), seed, draw0, _ptr(cent), _ptr(pick),
                               _ptr(ws), ws_bytes, _stream(stream))
    return _check(s, "kb_seed_dsquared", check)


def kb_cluster_diameter(batch, X, assign, diam, ws, ws_bytes, stream=None, check=True):
    s = lib().kb_cluster_diameter(ctypes.byref(batch), _ptr(X), _ptr(assign), _ptr(diam), _ptr(ws),
                                  ws_bytes, _stream(stream))
    return _check(s, "kb_cluster_diameter", check)


def kb_version() -> str:
    return lib().kb_version().decode()


# ---------------------------------------------------------------------------
# Convenience: device buffers for one batch.  Allocation and copies only.

class DeviceBatch:
    """Uploads the arrays of a synth.Batch-like object (numpy attributes) to the
    GPU and allocates every output and the workspace.  Holds the kb_batch /
    kb_params / kb_round_io structs that point into those tensors."""

    def __init__(self, b, device="cuda:0", iters=None, scorer=KB_SCORER_DEFAULT, stop_early=0):
        import numpy as np
        import torch
        self.torch = torch
        dev = torch.device(device)
        self.device = dev
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        self.seg_off = up(b.seg_off.astype(np.int32))
        self.koff = up(b.koff.astype(np.int32))
        self.X = up(b.X)
        self.flops = up(b.flops)
        self.bytes_ = up(b.bytes_)
        self.incumbent = up(b.incumbent)
        self.visits = up(b.visits)
        self.rsum = up(b.rsum)
        self.t = up(b.t.astype(np.int64))
        G, D, S, N, Ksum = b.G, b.D, b.S, b.N, b.Ksum
        self.G, self.D, self.S, self.N, self.Ksum = G, D, S, N, Ksum
        z = lambda shape, dt: torch.zeros(shape, dtype=dt, device=dev)
        self.bound = z((N,), torch.float32)
        self.alive = z((N,), torch.uint8)
        self.assign = z((N,), torch.int32)
        self.cent = z((Ksum, D), torch.float32)
        self.cent2 = z((Ksum, D), torch.float32)
        self.counts = z((Ksum,), torch.int32)
        self.objective = z((G,), torch.float32)
        self.Ncs = z((Ksum, S), torch.int32)
        self.mu = z((Ksum, S), torch.float32)
        self.ucb = z((Ksum, S), torch.float32)
        self.sel = z((G, 3), torch.int32)
        self.ksel = z((G,), torch.int32)
        self.rep = z((Ksum,), torch.int32)
        self.radius = z((Ksum,), torch.float32)
        self.diam = z((Ksum,), torch.float32)
        self.M = z((Ksum, S), torch.uint8)
        self.nvalid = z((G,), torch.int32)
        self.batch = make_batch(G, D, S, N, b.Kmax, Ksum, b.Nmax, self.seg_off, self.koff)
        self.params = make_params(b.peak_flops, b.peak_bw, b.c, b.prior_n, b.prior_mu,
                                  b.iters if iters is None else iters, scorer, stop_early)
        self.ws_bytes = kb_workspace_bytes(self.batch, self.params)
        self.ws = z((max(self.ws_bytes, 256),), torch.uint8)
        self.io = kb_round_io(*[_ptr(x) for x in (
            self.X, self.flops, self.bytes_, self.incumbent, self.visits, self.rsum, self.t,
            self.bound, self.alive, self.assign, self.cent, self.counts, self.objective,
            self.Ncs, self.mu, self.ucb, self.sel)])

    # the calls, on the buffers held here
    def prune(self, **kw):
        return kb_prune(self.batch, self.params, self.flops, self.bytes_, self.incumbent,
                        self.bound, self.alive, **kw)

    def cluster_step(self, cent_in, cent_out=None, **kw):
        return kb_cluster_step(self.batch, self.X, cent_in,
                               self.assign, self.cent if cent_out is None else cent_out,
                               self.counts, self.objective, self.ws, self.ws_bytes, **kw)

    def cluster_one(self, cent_in, **kw):
        """One Lloyd step through kb_cluster (iters = 1, cent_init = cent_in), which
        unlike kb_cluster_step honours params.scorer."""
        p = kb_params.from_buffer_copy(self.params)
        p.iters = 1
        return kb_cluster(self.batch, p, self.X, cent_in, self.assign, self.cent, self.counts,
                          self.objective, self.ws, self.ws_bytes, **kw)

    def cluster(self, cent_init=None, **kw):
        return kb_cluster(self.batch, self.params, self.X, cent_init, self.assign, self.cent,
                          self.counts, self.objective, self.ws, self.ws_bytes, **kw)

    def ucb_select(self, **kw):
        return kb_ucb_select(self.batch, self.params, self.assign, self.alive, self.bound,
                             self.visits, self.rsum, self.t, self.Ncs, self.mu, self.ucb,
                             self.sel, self.ws, self.ws_bytes, **kw)

    def sample(self, seed, draw, tau=1.0, alive=True, **kw):
        return kb_sample(self.batch, kb_sample_params(seed, draw, tau), self.assign,
                         self.alive if alive else None, self.bound, self.incumbent, self.sel,
                         self.ksel, self.ws, self.ws_bytes, **kw)

    def cluster_geometry(self, **kw):
        return kb_cluster_geometry(self.batch, self.X, self.cent, self.assign, self.rep,
                                   self.radius, self.ws, self.ws_bytes, **kw)

    def seed_farthest(self, cent=None, pick=True, **kw):
        return kb_seed_farthest(self.batch, self.X, self.cent2 if cent is None else cent,
                                self.rep if pick else None, self.ws, self.ws_bytes, **kw)

    def seed_dsquared(self, seed, draw0, cent=None, pick=True, **kw):
        return kb_seed_dsquared(self.batch, self.X, seed, draw0,
                                self.cent2 if cent is None else cent,
                                self.rep if pick else None, self.ws, self.ws_bytes, **kw)

    def cluster_diameter(self, **kw):
        return kb_cluster_diameter(self.batch, self.X, self.assign, self.diam, self.ws,
                                   self.ws_bytes, **kw)

    def round(self, **kw):
        return kb_round(self.batch, self.params, self.io, self.ws, self.ws_bytes, **kw)

    def iterate(self, ip: kb_iterate_params, h, target, reward, ok, sel_log, ksel_log, alive=None,
                **kw):
        """kb_iterate on the buffers held here (h, target, reward, ok, the logs: device
        tensors of the caller)."""
        io = kb_iterate_io(*[_ptr(x) for x in (
            self.X, h, target, alive, reward, ok, self.visits, self.rsum, self.t, self.assign,
            self.cent, self.counts, self.objective, self.rep, self.radius, self.M, self.nvalid,
            self.Ncs, self.mu, self.ucb, sel_log, ksel_log)])
        return kb_iterate(self.batch, self.params, ip, io, self.ws, self.ws_bytes, **kw)

    def host(self, name):
        return getattr(self, name).cpu().numpy()
