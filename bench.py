"""Benchmark of the arm-scoring round (prune -> cluster -> UCB select).

A step is one kb_round over one batch of synthetic traces, inputs resident in
HBM.  Prints ONE JSON line: whole-job candidate traces scored per second, the
roofline of the dominant kernel (the fused Lloyd kernel) measured with HIP
events, and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def lloyd_algorithmic_bytes(b, iters):
    """Streaming byte model of `iters` Lloyd steps: every step reads each
    candidate's D features and writes its 4-byte assignment, and reads and writes
    each search's centroids (2 * 4*K*D) and writes its counts (4*K)."""
    import numpy as np
    per_step = b.N * (4 * b.D + 4) + int(np.sum(np.diff(b.koff))) * (8 * b.D + 4)
    return iters * per_step


def measured_traffic(config):
    """HBM bytes per launch of the fused Lloyd kernel from the rocprofv3 --pmc runs
    recorded in profiles/traffic_config5.json, or None when the kernel source has
    changed since they were taken (or the workload is not config 5)."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "traffic_config5.json")
    if not os.path.exists(path) or config != 5:
        return None
    rec = json.load(open(path))
    h = hashlib.sha256()
    for name in ("kb_cluster.hip", "kb_cluster_dev.h"):      # the kernel and its device helpers
        h.update(open(os.path.join(ROOT, "paper_2511_18868_amd", "csrc", name), "rb").read())
    return rec["bytes_per_launch"] if rec.get("kernel_source_sha256") == h.hexdigest() else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="workload: benchmark configuration 1..5")
    ap.add_argument("--searches", type=int, default=0, help="override the number of searches (config 3/5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calib", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy three times (reference "
                         "for scaling the FETCH_SIZE / WRITE_SIZE counters of a --pmc run)")
    ap.add_argument("--no-step", action="store_true",
                    help="skip the single-Lloyd-step timing (so a kernel trace of this run holds "
                         "only full kb_cluster launches of the fused kernel)")
    ap.add_argument("--no-loop-steps", action="store_true",
                    help="skip the timings of the steps outside the round (draw, representatives, "
                         "paper-form mask, masked selection, statistics update)")
    ap.add_argument("--cpu-sample", type=int, default=0, help="searches in the CPU baseline sample")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU; --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2511_18868_amd import binding as kb, synth

    kb.lib()   # fail loudly if the HIP library is missing
    kw = {}
    if args.searches and args.config in (3, 5):
        kw["G"] = args.searches
    t0 = time.time()
    b = synth.make(args.config, **kw)
    gen_s = time.time() - t0
    d = kb.DeviceBatch(b, device="cuda:0")
    torch.cuda.synchronize()

    if args.copy_calib:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

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

    # per-stage times with HIP events on the stream the kernels run on
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

    reps = max(3, min(args.steps, 20))
    d.round()
    torch.cuda.synchronize()
    cl_mean, cl_med = timed(d.cluster, reps)
    pr_mean, _ = timed(d.prune, reps)
    uc_mean, _ = timed(d.ucb_select, reps)
    step_mean = float("nan")
    modes = {}
    if not args.no_step:
        d.cent2.copy_(d.cent)
        step_mean, _ = timed(lambda: d.cluster_step(d.cent2), reps)
        # the same clustering with every tile scored in every step (no distance
        # bounds), on the matrix cores and on the vector ALU
        for name, mode in (("matrix_cores_every_tile", 2), ("vector_alu_every_tile", 1)):
            kb.kb_set_scorer(mode)
            d.cluster()
            torch.cuda.synchronize()
            modes[name] = round(timed(d.cluster, max(3, reps // 2))[0], 4)
        kb.kb_set_scorer(0)

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
        # optional farthest-point seeding: K_g dependent passes over the rows of every
        # search, which stay on chip
        loop["seed_farthest"] = timed(d.seed_farthest, 3)[0]
        loop["seed_dsquared"] = timed(lambda: d.seed_dsquared(20251118, 0), 3)[0]
        loop = {k: round(v, 4) for k, v in loop.items()}
        nk_rows = float(np.sum(np.diff(b.seg_off).astype(np.float64) * np.diff(b.koff)))
        # four fp64-rate vector instructions (widen, subtract, multiply, add) per feature,
        # row and pass against 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz
        loop["seed_farthest_fp64_frac"] = round(
            nk_rows * 4 * b.D / (loop["seed_farthest"] * 1e-3) / (256 * 4 * 16 * 2.4e9), 3)
        # representatives: every feature row and assignment read once
        loop["cluster_geometry_GBs"] = round(
            b.N * (4 * b.D + 4) / (loop["cluster_geometry"] * 1e-3) / 1e9, 1)
        # the draw reads the 4-byte assignment of every candidate (mask and bound only of
        # the members of the chosen cluster)
        loop["sample_GBs"] = round(b.N * 4 / (loop["sample"] * 1e-3) / 1e9, 1)

    lloyd_bytes = lloyd_algorithmic_bytes(b, b.iters)
    achieved = lloyd_bytes / (cl_mean * 1e-3) / 1e9
    big = b.Kmax > 64 or b.Nmax > 65536
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": measured_traffic(args.config),
                "kernel": "kb_cluster launch sequence (multi-workgroup path)" if big
                          else "cluster_fused_kernel",
                "ms": round(cl_mean, 4), "algorithmic_bytes": lloyd_bytes}
    # distance contraction: 2*N_g*K_g*D flops per step, 3 bf16 products issued per flop
    nk = float(np.sum(np.diff(b.seg_off).astype(np.float64) * np.diff(b.koff)))
    logical = 2.0 * nk * b.D * b.iters
    mfma = {"logical_TFLOPs": round(logical / (cl_mean * 1e-3) / 1e12, 1),
            "issued_bf16_TFLOPs_if_every_tile_scored": round(3 * logical / (cl_mean * 1e-3) / 1e12, 1),
            "bf16_peak_TFLOPs": 2500.0}

    out = {
        "metric": "candidate traces scored/sec per round",
        "value": round(value, 1), "unit": "traces/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config{args.config} full kb_round", "G": b.G, "N": b.N,
                   "D": b.D, "S": b.S, "Ksum": b.Ksum, "Kmax": b.Kmax, "iters": b.iters,
                   "lloyd_mode": "matrix cores + distance bounds (library default; results "
                                 "identical to scoring every tile)"},
        "stages_ms": {"prune": round(pr_mean, 4), "cluster": round(cl_mean, 4),
                      "ucb_select": round(uc_mean, 4),
                      "one_lloyd_step": None if args.no_step else round(step_mean, 4)},
        "cluster_ms_other_modes": modes,
        "iteration_steps_ms": loop,
        "lloyd_step_GBs": None if args.no_step else round(
            lloyd_algorithmic_bytes(b, 1) / (step_mean * 1e-3) / 1e9, 1),
        "round_streaming_GBs": round(
            (lloyd_bytes + b.N * 13 + b.N * (8 * b.S + 9)) / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline": roofline,
        "distance_contraction": mfma,
        "input_generation_s": round(gen_s, 1),
    }

    if not args.no_cpu_baseline:
        import copy
        import oracle
        # bounded sample: the first `gs` searches of the same batch
        gs = args.cpu_sample or max(1, min(b.G, {1: 1, 2: 1, 3: 1024, 4: 1, 5: 4096}[args.config]))
        sb = copy.copy(b)
        sb.G = gs
        sb.seg_off = b.seg_off[:gs + 1]
        sb.koff = b.koff[:gs + 1]
        n, ks = int(sb.seg_off[-1]), int(sb.koff[-1])
        sb.X, sb.flops, sb.bytes_ = b.X[:n], b.flops[:n], b.bytes_[:n]
        sb.visits, sb.rsum = b.visits[:n], b.rsum[:n]
        sb.incumbent, sb.t = b.incumbent[:gs], b.t[:gs]
        iters = b.iters
        if args.config == 4:
            iters = 1     # one Lloyd step of the single large search, see `sample`
        t0 = time.perf_counter()
        oracle.round_(sb, iters=iters)
        cdt = time.perf_counter() - t0
        scale = b.iters / iters
        out["cpu_baseline"] = {
            "value": round(n / (cdt * scale), 1), "unit": "traces/s",
            "cores": oracle.max_threads() if gs > 1 else 1, "kind": "oracle",
            "sample": f"first {gs} of {b.G} searches ({n} of {b.N} candidates), full round"
                      + (f", {iters} of {b.iters} Lloyd steps timed and scaled" if scale != 1 else ""),
            "seconds": round(cdt, 2)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
