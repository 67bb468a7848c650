"""Benchmark of the arm-scoring round (prune -> cluster -> UCB select).

A step is one kb_round over one batch of synthetic traces, inputs resident in
HBM.  Prints ONE JSON line: whole-job candidate traces scored per second, the
roofline of the dominant kernel (the Lloyd clustering) measured with HIP
events, the other benchmark configurations timed in the same run, and the CPU
oracle timed on the host cores.
"""
import argparse
import ctypes
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
BF16_PEAK_TFLOPS = 2500.0
FP32_VECTOR_PEAK_TFLOPS = 78.6      # unpacked fp32 fused multiply-adds (packed forms are not used)


def lloyd_step_bytes(b):
    """Streaming byte model of ONE Lloyd step: read each candidate's D features, write
    its 4-byte assignment; read and write each search's centroids (2 * 4*K*D), write
    its counts (4*K).  Also the compulsory traffic of a whole kb_cluster call: no
    implementation can do with less than one pass over the features."""
    return b.N * (4 * b.D + 4) + b.Ksum * (8 * b.D + 4)


def measured_traffic(config):
    """HBM bytes per kb_cluster call from the rocprofv3 --pmc runs recorded in
    profiles/traffic_config<n>.json, or None when there is no record or the kernel
    sources have changed since the counters were taken."""
    path = os.path.join(ROOT, "profiles", f"traffic_config{config}.json")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path))
    h = hashlib.sha256()
    for name in rec.get("sources", []):
        h.update(open(os.path.join(ROOT, "paper_2511_18868_amd", "csrc", name), "rb").read())
    return rec if rec.get("kernel_source_sha256") == h.hexdigest() else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=5, help="workload: benchmark configuration 1..5")
    ap.add_argument("--searches", type=int, default=0, help="override the number of searches (config 3/5)")
    ap.add_argument("--scorer", type=int, default=0, help="kb_params.scorer of the timed rounds")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the timings of the other benchmark configurations")
    ap.add_argument("--no-step", action="store_true",
                    help="skip the single-Lloyd-step and other-scorer timings (so a kernel trace of "
                         "this run holds only full kb_cluster calls in the chosen mode)")
    ap.add_argument("--no-loop-steps", action="store_true",
                    help="skip the timings of the steps outside the round (draw, representatives, "
                         "paper-form mask, masked selection, statistics update, seeding)")
    ap.add_argument("--cpu-sample", type=int, default=0, help="searches in the CPU baseline sample")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU; --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2511_18868_amd import binding as kb, synth

    kb.lib()   # fail loudly if the HIP library is missing
    dev = "cuda:0"

    # per-call times with HIP events on the stream the kernels run on (torch's
    # current stream, which the binding hands to the library)
    def timed(fn, reps):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(reps)]
        for s, e in ev:
            s.record()
            fn()
            e.record()
        torch.cuda.synchronize()
        ts = sorted(s.elapsed_time(e) for s, e in ev)
        return float(np.mean(ts)), float(ts[len(ts) // 2])

    # plain device-to-device copy of 1 GiB: the practical HBM ceiling of this machine (and
    # the reference that scales the FETCH_SIZE / WRITE_SIZE counters of a --pmc run)
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    torch.cuda.synchronize()
    copy_ms, _ = timed(lambda: dst.copy_(src), 5)
    copy_GBs = 2.0 * src.numel() * 4 / (copy_ms * 1e-3) / 1e9
    del src, dst
    torch.cuda.empty_cache()

    kw = {}
    if args.searches and args.config in (3, 5):
        kw["G"] = args.searches
    t0 = time.time()
    b = synth.make(args.config, **kw)
    gen_s = time.time() - t0
    d = kb.DeviceBatch(b, device=dev, scorer=args.scorer)
    torch.cuda.synchronize()

    for _ in range(args.warmup):
        d.round()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        d.round()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = b.N / (dt / args.steps)

    reps = max(3, min(args.steps, 20))
    d.round()
    torch.cuda.synchronize()
    cl_mean, cl_med = timed(d.cluster, reps)
    pr_mean, _ = timed(d.prune, reps)
    uc_mean, _ = timed(d.ucb_select, reps)
    step_mean = None
    modes = {}
    if not args.no_step:
        d.cent2.copy_(d.cent)
        step_mean, _ = timed(lambda: d.cluster_step(d.cent2), reps)
        # the same clustering with every candidate scored in every step, on the matrix
        # cores and on the vector ALU (identical results, see kb_params.scorer)
        for name, mode in (("matrix_cores_every_candidate", 2), ("vector_alu_every_candidate", 1)):
            dm = kb.make_params(b.peak_flops, b.peak_bw, b.c, b.prior_n, b.prior_mu, b.iters, mode)
            run = lambda: kb.kb_cluster(d.batch, dm, d.X, None, d.assign, d.cent, d.counts,
                                        d.objective, d.ws, d.ws_bytes)
            run()
            torch.cuda.synchronize()
            modes[name] = round(timed(run, max(3, reps // 2))[0], 4)
        # ... and the default mode with kb_params.stop_early: searches stop at their first
        # step without a move (same outputs; not the timed round, which runs every step)
        ds = kb.make_params(b.peak_flops, b.peak_bw, b.c, b.prior_n, b.prior_mu, b.iters, args.scorer, 1)
        run = lambda: kb.kb_cluster(d.batch, ds, d.X, None, d.assign, d.cent, d.counts,
                                    d.objective, d.ws, d.ws_bytes)
        run()
        torch.cuda.synchronize()
        modes["default_stop_early"] = round(timed(run, max(3, reps // 2))[0], 4)
        d.cluster()

    # the remaining device-side steps of an iteration of Alg. 1 (not part of the
    # timed round): in-cluster draw, cluster representatives, the paper-form mask,
    # selection under it, the draw with the paper's potential, statistics update
    loop = {}
    if not args.no_loop_steps:
        R = 3
        h, target, theta = synth.signatures(b, R)
        reward, okv = synth.feedback(b)
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(d.device)
        dh, dtg, drw, dok = up(h), up(target), up(reward), up(okv)
        d.round()
        sp = kb.kb_sample_params(20251118, 1, 1.0)
        loop["sample"] = timed(lambda: d.sample(20251118, 1, 1.0), reps)[0]
        loop["cluster_geometry"] = timed(d.cluster_geometry, reps)[0]
        loop["strategy_mask"] = timed(lambda: kb.kb_strategy_mask(
            d.batch, R, dh, dtg, d.rep, theta, d.M, d.nvalid), reps)[0]
        loop["ucb_select_masked"] = timed(lambda: kb.kb_ucb_select_masked(
            d.batch, d.params, d.assign, None, None, d.M, d.visits, d.rsum, d.t, d.Ncs, d.mu, d.ucb,
            d.sel, d.ws, d.ws_bytes), reps)[0]
        loop["sample_signature"] = timed(lambda: kb.kb_sample_signature(
            d.batch, sp, d.assign, None, R, dh, dtg, theta, d.sel, d.ksel, d.ws, d.ws_bytes), reps)[0]
        loop["update_stats"] = timed(lambda: kb.kb_update_stats(
            d.batch, d.params, d.sel, d.ksel, drw, dok, d.visits, d.rsum, d.Ncs, d.mu, d.t), reps)[0]
        loop["cluster_diameter"] = timed(d.cluster_diameter, 3)[0]
        loop["seed_farthest"] = timed(d.seed_farthest, 3)[0]
        loop["seed_dsquared"] = timed(lambda: d.seed_dsquared(20251118, 0), 3)[0]
        # ten whole iterations of Alg. 1 in one call (re-clustering in the first, warm start)
        T = 10
        fb = [synth.feedback(b, seed=r) for r in range(T)]
        drw10 = up(np.stack([f[0] for f in fb]))
        dok10 = up(np.stack([f[1] for f in fb]))
        sl = torch.zeros((T, b.G, 3), dtype=torch.int32, device=d.device)
        kl = torch.zeros((T, b.G), dtype=torch.int32, device=d.device)
        ipar = kb.kb_iterate_params(T, 10, 0, 1, R, theta, sp)
        loop["iterate_10_rounds"] = timed(lambda: d.iterate(ipar, dh, dtg, drw10, dok10, sl, kl), 3)[0]
        del drw10, dok10, sl, kl
        loop = {k: round(v, 4) for k, v in loop.items()}
        nk_rows = float(np.sum(np.diff(b.seg_off).astype(np.float64) * np.diff(b.koff)))
        # four fp64-rate vector instructions (widen, subtract, multiply, add) per feature,
        # row and pass against 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz
        loop["seed_farthest_fp64_frac"] = round(
            nk_rows * 4 * b.D / (loop["seed_farthest"] * 1e-3) / (256 * 4 * 16 * 2.4e9), 3)
        loop["cluster_geometry_GBs"] = round(
            b.N * (4 * b.D + 4) / (loop["cluster_geometry"] * 1e-3) / 1e9, 1)
        loop["sample_GBs"] = round(b.N * 4 / (loop["sample"] * 1e-3) / 1e9, 1)

    # ---- roofline of the dominant kernel: the Lloyd clustering of the round
    big = b.Kmax > 64 or b.Nmax > 65536
    step_bytes = lloyd_step_bytes(b)
    model_bytes = step_bytes * b.iters
    rec = measured_traffic(args.config) if args.scorer == 0 else None
    traffic = rec["bytes_per_launch"] if rec else None
    if traffic is not None:
        moved, basis = traffic, "HBM bytes from FETCH_SIZE / WRITE_SIZE counters (profiles/)"
    else:
        moved, basis = step_bytes, "compulsory bytes (one pass over the features): a lower bound"
    achieved = moved / (cl_mean * 1e-3) / 1e9
    roofline = {
        "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
        "basis": basis,
        "frac_of_measured_copy_rate": round(achieved / copy_GBs, 4),
        "kernel": "kb_cluster launch sequence (multi-workgroup path)" if big else "cluster_fused_kernel",
        "ms": round(cl_mean, 4),
        "compulsory_bytes": step_bytes,
        "traffic_over_compulsory": None if traffic is None else round(traffic / step_bytes, 2),
        # the streaming model charges every candidate in every step; the default mode
        # leaves most of them unread, so this is a work rate, not a fraction of the peak
        "model_bytes_every_step": model_bytes,
        "model_GBs": round(model_bytes / (cl_mean * 1e-3) / 1e9, 1),
    }
    # scorer mode 2 is the streaming Lloyd iteration of the byte model: every candidate
    # is read in every step
    if rec and rec.get("bytes_per_launch_every_candidate") and "matrix_cores_every_candidate" in modes:
        t2, ms2 = rec["bytes_per_launch_every_candidate"], modes["matrix_cores_every_candidate"]
        roofline["every_candidate_mode"] = {
            "ms": ms2, "traffic": t2, "achieved": round(t2 / (ms2 * 1e-3) / 1e9, 1),
            "frac": round(t2 / (ms2 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "frac_of_measured_copy_rate": round(t2 / (ms2 * 1e-3) / 1e9 / copy_GBs, 4)}
    # distance contraction: 2*N_g*K_g*D flops per step; the matrix-core scorer issues
    # three bf16 products per term
    nk = float(np.sum(np.diff(b.seg_off).astype(np.float64) * np.diff(b.koff)))
    logical = 2.0 * nk * b.D * b.iters
    mfma = {"logical_TFLOPs": round(logical / (cl_mean * 1e-3) / 1e12, 1),
            "bf16_peak_TFLOPs": BF16_PEAK_TFLOPS}
    if big:
        # the multi-workgroup path scores every candidate in every step
        mfma["issued_bf16_TFLOPs"] = round(3 * logical / (cl_mean * 1e-3) / 1e12, 1)
        mfma["mfma_frac_whole_call"] = round(3 * logical / (cl_mean * 1e-3) / 1e12 / BF16_PEAK_TFLOPS, 4)

    out = {
        "metric": "candidate traces scored/sec per round",
        "value": round(value, 1), "unit": "traces/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config{args.config} full kb_round", "G": b.G, "N": b.N,
                   "D": b.D, "S": b.S, "Ksum": b.Ksum, "Kmax": b.Kmax, "iters": b.iters,
                   "scorer": args.scorer},
        "stages_ms": {"prune": round(pr_mean, 4), "cluster": round(cl_mean, 4),
                      "ucb_select": round(uc_mean, 4),
                      "one_lloyd_step": None if step_mean is None else round(step_mean, 4)},
        "cluster_ms_other_scorers": modes,
        "iteration_steps_ms": loop,
        "lloyd_step_GBs": None if step_mean is None else round(
            step_bytes / (step_mean * 1e-3) / 1e9, 1),
        "lloyd_step_frac_of_hbm_peak": None if step_mean is None else round(
            step_bytes / (step_mean * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "copy_GBs": round(copy_GBs, 1),
        "roofline": roofline,
        "distance_contraction": mfma,
        "input_generation_s": round(gen_s, 1),
    }
    del d
    torch.cuda.empty_cache()

    # ---- the other benchmark configurations, timed the same way in the same run
    if not args.no_configs:
        cfgs = {}
        for c in (1, 2, 3, 4, 5):
            if c == args.config:
                continue
            bc = synth.make(c)
            dc = kb.DeviceBatch(bc, device=dev)
            for _ in range(3):
                dc.round()
            torch.cuda.synchronize()
            n = 50 if c <= 3 else 20
            r_mean, r_med = timed(dc.round, n)
            c_mean, _ = timed(dc.cluster, n)
            dcs = kb.make_params(bc.peak_flops, bc.peak_bw, bc.c, bc.prior_n, bc.prior_mu, bc.iters, 0, 1)
            stop_run = lambda: kb.kb_cluster(dc.batch, dcs, dc.X, None, dc.assign, dc.cent, dc.counts,
                                             dc.objective, dc.ws, dc.ws_bytes)
            stop_run()
            torch.cuda.synchronize()
            cs_mean, _ = timed(stop_run, n)
            dc.cluster()
            # the same round recorded once into a HIP graph and replayed (the library only
            # enqueues kernels, so a call can be captured)
            side, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                dc.round()
            graph.replay()
            torch.cuda.synchronize()
            _, g_med = timed(graph.replay, n)
            e = {"N": bc.N, "G": bc.G, "D": bc.D, "Kmax": bc.Kmax, "S": bc.S, "iters": bc.iters,
                 "round_ms": round(r_med, 4), "cluster_ms": round(c_mean, 4),
                 "cluster_ms_stop_early": round(cs_mean, 4),
                 "round_ms_graph_replay": round(g_med, 4),
                 "traces_per_s": round(bc.N / (r_med * 1e-3), 1)}
            del graph
            sb = lloyd_step_bytes(bc)
            if c in (1, 2):
                # one search on one workgroup: launch and barrier latency, not bandwidth
                e["bound"] = "latency"
                e["round_us"] = round(r_med * 1e3, 1)
                e["us_per_lloyd_step"] = round(c_mean * 1e3 / bc.iters, 2)
            elif c == 3:
                e["bound"] = "hbm"
                e["inputs_cache_resident"] = True   # 200 MB of inputs: repeats are partly served by the 256 MB Infinity Cache
                e["model_GBs"] = round(sb * bc.iters / (c_mean * 1e-3) / 1e9, 1)
                e["compulsory_frac_of_hbm_peak"] = round(sb / (c_mean * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
            else:
                flops = 2.0 * bc.N * bc.Kmax * bc.D * bc.iters
                e["bound"] = "mfma"
                e["issued_bf16_TFLOPs"] = round(3 * flops / (c_mean * 1e-3) / 1e12, 1)
                e["mfma_frac_whole_call"] = round(3 * flops / (c_mean * 1e-3) / 1e12 / BF16_PEAK_TFLOPS, 4)
                pv = kb.make_params(bc.peak_flops, bc.peak_bw, bc.c, bc.prior_n, bc.prior_mu, bc.iters,
                                    kb.KB_SCORER_VECTOR_ALU)
                runv = lambda: kb.kb_cluster(dc.batch, pv, dc.X, None, dc.assign, dc.cent, dc.counts,
                                             dc.objective, dc.ws, dc.ws_bytes)
                runv()
                torch.cuda.synchronize()
                v_mean, _ = timed(runv, 3)
                e["cluster_ms_fp32_vector_alu"] = round(v_mean, 4)
                e["fp32_vector_TFLOPs"] = round(flops / (v_mean * 1e-3) / 1e12, 1)
                e["fp32_vector_frac_of_peak"] = round(flops / (v_mean * 1e-3) / 1e12 / FP32_VECTOR_PEAK_TFLOPS, 4)
                e["matrix_over_vector_speedup"] = round(v_mean / c_mean, 2)
            cfgs[f"config{c}"] = e
            del dc, bc
            torch.cuda.empty_cache()
        # the scale the paper itself runs: 183 searches of 12-41 candidates, 5 features,
        # K = 3, |S| = 6, ten Lloyd steps
        bp = synth.paper_scale()
        dp = kb.DeviceBatch(bp, device=dev)
        for _ in range(3):
            dp.round()
        torch.cuda.synchronize()
        _, p_med = timed(dp.round, 50)
        cfgs["paper_scale"] = {"N": bp.N, "G": bp.G, "D": bp.D, "Kmax": bp.Kmax, "S": bp.S,
                               "iters": bp.iters, "round_us": round(p_med * 1e3, 1), "bound": "latency"}
        # twenty whole iterations of Alg. 1 in one call, re-clustering every tenth
        Rp, Tp = 3, 20
        hp, tgp, thp = synth.signatures(bp, Rp)
        fbp = [synth.feedback(bp, seed=r) for r in range(Tp)]
        upp = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        dhp, dtp = upp(hp), upp(tgp)
        drp, dop = upp(np.stack([f[0] for f in fbp])), upp(np.stack([f[1] for f in fbp]))
        slp = torch.zeros((Tp, bp.G, 3), dtype=torch.int32, device=dev)
        klp = torch.zeros((Tp, bp.G), dtype=torch.int32, device=dev)
        ipp = kb.kb_iterate_params(Tp, 10, 0, 1, Rp, thp, kb.kb_sample_params(20251118, 1, 1.0))
        itp = lambda: dp.iterate(ipp, dhp, dtp, drp, dop, slp, klp)
        itp()
        torch.cuda.synchronize()
        cfgs["paper_scale"]["iteration_us"] = round(timed(itp, 10)[1] * 1e3 / Tp, 1)
        del dp, bp
        out["configs"] = cfgs

    if not args.no_cpu_baseline:
        import copy
        import oracle

        def subset(gs):
            sb = copy.copy(b)
            sb.G = gs
            sb.seg_off = b.seg_off[:gs + 1]
            sb.koff = b.koff[:gs + 1]
            n, ks = int(sb.seg_off[-1]), int(sb.koff[-1])
            sb.X, sb.flops, sb.bytes_ = b.X[:n], b.flops[:n], b.bytes_[:n]
            sb.visits, sb.rsum = b.visits[:n], b.rsum[:n]
            sb.incumbent, sb.t = b.incumbent[:gs], b.t[:gs]
            return sb, n

        # bounded sample: the first `gs` searches of the same batch
        gs = args.cpu_sample or max(1, min(b.G, {1: 1, 2: 1, 3: 1024, 4: 1, 5: 4096}[args.config]))
        sb, n = subset(gs)
        iters = 1 if args.config == 4 else b.iters   # one Lloyd step of the single large search
        t0 = time.perf_counter()
        oracle.round_(sb, iters=iters)
        cdt = time.perf_counter() - t0
        scale = b.iters / iters
        cores = oracle.max_threads() if gs > 1 else 1
        out["cpu_baseline"] = {
            "value": round(n / (cdt * scale), 1), "unit": "traces/s",
            "cores": cores, "kind": "oracle",
            "sample": f"first {gs} of {b.G} searches ({n} of {b.N} candidates), full round"
                      + (f", {iters} of {b.iters} Lloyd steps timed and scaled" if scale != 1 else ""),
            "seconds": round(cdt, 2)}
        if gs > 1:
            # the same oracle on one host thread, on a smaller sample
            g1 = max(1, gs // 16)
            s1, n1 = subset(g1)
            omp = ctypes.CDLL("libgomp.so.1")
            omp.omp_set_num_threads(1)
            t0 = time.perf_counter()
            oracle.round_(s1, iters=iters)
            c1 = time.perf_counter() - t0
            omp.omp_set_num_threads(cores)
            out["cpu_baseline"]["single_thread"] = {
                "value": round(n1 / (c1 * scale), 1), "unit": "traces/s", "cores": 1,
                "sample": f"first {g1} searches ({n1} candidates), full round", "seconds": round(c1, 2)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
