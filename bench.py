#!/usr/bin/env python3
"""Benchmark of the Barnes-Hut t-SNE gradient step on one MI355X.

A "step" is one full iteration of Alg. 1 lines 4-8 (tree build, walk + Z, attractive forces over
the CSR P, update) through the C ABI, with X, P and Y resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5|cfg4|cfg3|cfg2|cfg1]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
STANDIN_D = 64                 # see workload_inputs()
STANDIN_MEAN_SCALE = 2.0
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "attract_cfg5_hbm_traffic.md")


def workload_inputs(name):
    """Synthetic X for the named configuration (recipes in paper_1807_11824_amd/synth.py).

    cfg5 is the headline configuration as stated: N = 1,281,167, D = 2048 (10.5 GB of X, about 20 s to draw on
    the host and 7 s for the exact tsne_build_P).  cfg5_standin is a quick substitute for kernel work: the same
    1000-cluster ReLU-Gaussian mixture drawn in D' = 64 dimensions with the cluster means at scale 2, which gives
    the same neighbourhood structure (every point's neighbours lie in its own cluster) in a second; it is never
    what the default run reports.
    """
    from paper_1807_11824_amd import synth
    if name == "cfg5_standin":
        c = dict(synth.CONFIGS["cfg5"])
        X, _ = synth.gaussian_mixture(c["n"], STANDIN_D, 1000, STANDIN_MEAN_SCALE, 1.0, seed=0, relu=True)
        c["d_used"] = STANDIN_D
        return X, c
    c = dict(synth.CONFIGS[name])
    if name == "cfg5":
        X, _ = synth.config5()
        c["d_used"] = c["d"]
    elif name == "cfg4":
        X, _ = synth.config4()
        c["d_used"] = c["d"]
    elif name == "cfg3":
        X, _ = synth.config3()
        c["d_used"] = c["d"]
    elif name == "cfg2":
        X, _ = synth.config2()
        c["d_used"] = c["d"]
    else:
        X, _ = synth.config1()
        c["d_used"] = c["d"]
    return X, c


def cpu_baseline(Y0, P_host, bits, X=None, cfg=None, P_gpu_seconds=None):
    """The CPU oracle as it stands, timed on this host: a few whole iterations of the same workload, and the
    construction of P (kNN in double precision, Eq. (1)) on a sample of rows, extrapolated to all rows."""
    import oracle
    pr = oracle.RunParams.default(bits=bits)
    n = Y0.shape[0]
    iters = 3 if n > 200_000 else 10
    t0 = time.time()
    oracle.run(Y0, P_host["row_ptr"], P_host["col"], P_host["val"], pr, iters)
    dt = time.time() - t0
    out = dict(value=iters / dt, unit="iterations/s", cores=oracle.threads(), kind="oracle",
               sample=f"{iters} full iterations (tree + walk + attraction + update) of the same N={n} workload from Y0")
    if X is not None:
        # neighbour search and Eq. (1) for a sample of query rows against all n rows; the symmetric CSR (a sort of
        # all n k entries) is not sampled
        k, perp = cfg["k"], cfg["perplexity"]
        rng = np.random.default_rng(0)
        probe = np.sort(rng.choice(n, 16, replace=False)).astype(np.int32)
        t0 = time.time()
        oracle.knn(X, k, rows=probe)
        t16 = time.time() - t0
        rows = int(min(256, max(16, 12.0 / max(t16 / 16, 1e-9))))      # about 12 s of work
        sample = np.sort(rng.choice(n, rows, replace=False)).astype(np.int32)
        t0 = time.time()
        _, d2 = oracle.knn(X, k, rows=sample)
        t_knn = time.time() - t0
        t0 = time.time()
        oracle.cond_p(d2, perp)
        t_cond = time.time() - t0
        est = (t_knn + t_cond) / rows * n
        out["build_P"] = dict(rows_sampled=rows, knn_s=t_knn, cond_p_s=t_cond, extrapolated_s_all_rows=est,
                              note="oracle kNN (sequential double-precision sums) + Eq. (1) on the sampled rows against "
                                   "all rows, scaled by n / rows; symmetrisation not included",
                              gpu_build_P_s=P_gpu_seconds)
    return out


def sweep(dev, overlap, sizes, n_iter, reorder_every, approx_tau=0, sweep_recall=False):
    """Stand-in for the paper's scaling experiment (Sec. IV-B: simulated 50-d data in four clusters): time of a
    whole run of n_iter iterations (exaggeration 12 for the first quarter), the phases of an iteration averaged
    over the run, and the time of tsne_build_P, as N grows.  Perplexity 30, k = 90, theta = 0.5.  With approx_tau > 0
    P comes from the inverted-file search (sqrt(N) lists, approx_tau probed), which is the paper's own first phase;
    the final KL divergence against that run's P and the objective's value are then not comparable between the two."""
    import torch
    from paper_1807_11824_amd import Tsne, build_P, build_P_approx, synth
    for n in sizes:
        X, _ = synth.gaussian_mixture(n, 50, 4, 10.0, 1.0, seed=0)
        Xd = torch.from_numpy(X).to(dev)
        del X
        torch.cuda.synchronize()
        t0 = time.time()
        recall = None
        if approx_tau > 0 and n > 90 * 8:
            P = build_P_approx(Xd, 30.0, 90, min(approx_tau, int(round(n ** 0.5))), want_knn=sweep_recall)
        else:
            P = build_P(Xd, 30.0, 90)
        torch.cuda.synchronize()
        t_build = time.time() - t0
        if sweep_recall and approx_tau > 0 and n > 90 * 8:
            # (untimed) recall of the approximate lists against the exact ones on 20,000 sampled rows
            ex = build_P(Xd, 30.0, 90, want_knn=True)
            rows = torch.randperm(n, device=dev, generator=torch.Generator(device=dev).manual_seed(0))[:20000]
            hit = (P["knn_idx"][rows].long()[:, :, None] == ex["knn_idx"][rows].long()[:, None, :]).any(-1)
            recall = float(hit.float().mean().item())
            del ex, hit
            P["knn_idx"] = P["knn_d2"] = None
        del Xd
        Yd = torch.from_numpy(synth.y0(n)).to(dev)
        ts = Tsne(n, overlap=overlap, max_nnz=P["nnz"], reorder_every=reorder_every, exaggeration_iters=n_iter // 4)
        t0 = time.time()
        ts.set_P(P["row_ptr"], P["col"], P["val"])
        torch.cuda.synchronize()
        t_setp = time.time() - t0
        ts.timing_begin((n_iter + 7) // 8, 8)
        t0 = time.time()
        ts.run(Yd, n_iter)
        torch.cuda.synchronize()
        dt = time.time() - t0
        tm = ts.timing_end()
        st = ts.status()
        ts.close()
        print(json.dumps({"workload": "50-d, 4 Gaussian clusters (means N(0, 10^2), sigma 1)", "n": n, "nnz": P["nnz"],
                          "n_iter": n_iter, "reorder_every": reorder_every, "approx_tau": approx_tau, "run_s": round(dt, 4),
                          "ms_per_step": dt / n_iter * 1e3, "iterations_per_s": n_iter / dt,
                          "phases_ms": {k[:-3]: round(v, 4) for k, v in tm.items() if k.endswith("_ms")},
                          "build_P_s": round(t_build, 4), "set_P_s": round(t_setp, 4), "status": st,
                          **({"recall_at_k": recall} if recall is not None else {})}), flush=True)
        del P, Yd


def step_bytes(n, m_cells, near, far, radix_passes):
    """Bytes one iteration has to move, kernel by kernel as implemented (N points, M tree cells; every array
    counted once per kernel that streams it, gathers that stay in cache not counted)."""
    b = {}
    b["sort"] = (8 + 8) * n + 8 * n * (radix_passes - 1) + 16 * n * radix_passes    # words written, digit counts, passes
    b["cells"] = (8 + 8 + 8 + 4 + 2) * n + (8 + 2 + 4 + 16) * n + 5 * m_cells + 8 * n + (5 + 32 + 32) * m_cells
    b["walk"] = (8 + 8 + 4) * n + 32 * m_cells
    b["attract"] = 6 * near + 8 * far + (4 + 4 + 8 + 8) * n
    b["update"] = 64 * n
    return b


def traffic_from_profile(nnz):
    """HBM bytes per step of the attraction kernels as counted by rocprofv3 (profiles/attract_cfg5_hbm_traffic.md
    holds a line 'TRAFFIC nnz=<entries of P> bytes=<bytes per step>'); None if no line matches this P."""
    try:
        for line in open(TRAFFIC_PROFILE):
            f = line.split()
            if len(f) >= 3 and f[0] == "TRAFFIC" and f[1] == f"nnz={nnz}":
                return float(f[2].split("=")[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg5", help="cfg5 (as stated, D = 2048) | cfg5_standin | cfg4 | cfg3 | cfg2 | cfg1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--overlap", type=int, default=1)
    ap.add_argument("--leaf-cap", type=int, default=8)
    ap.add_argument("--no-full-run", action="store_true", help="skip the separate 1000-iteration run (profiling)")
    ap.add_argument("--no-standalone", action="store_true",
                    help="skip the serial re-timing of the kernels on their own (profiling: every launch a profiler "
                         "then sees belongs to warm-up or timed steps)")
    ap.add_argument("--knn-rows", type=int, default=0,
                    help="profiling aid: build P from the first R rows of the workload's X and exit (counter runs of the "
                         "neighbour-search kernels on a subset; prints seconds and nnz)")
    ap.add_argument("--P-cache", default="",
                    help="profiling aid: a path prefix; if <prefix>.npz exists P is loaded from it (X is neither drawn "
                         "nor searched, build_P_s is reported as null), otherwise P is built as usual and saved there")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark: the paper's synthetic scaling workload (50-d, 4 Gaussian clusters, "
                         "Sec. IV-B) at N = 500 ... 5M, one JSON line per N")
    ap.add_argument("--sweep-n", default="500,1000,2000,4000,8000,16000,32000,64000,128000,512000,2000000,5000000")
    ap.add_argument("--sweep-iters", type=int, default=1000)
    ap.add_argument("--reorder-every", type=int, default=0, help="--sweep only: tsne_params.reorder_every")
    ap.add_argument("--sweep-approx-tau", type=int, default=0,
                    help="--sweep only: build P with tsne_build_P_approx, this many lists probed (0 = exact)")
    ap.add_argument("--sweep-recall", action="store_true",
                    help="--sweep with --sweep-approx-tau: also build the exact lists (untimed) and report recall at k")
    ap.add_argument("--approx-tau", type=int, default=4,
                    help="also time tsne_build_P_approx (inverted-file neighbour search, sqrt(N) lists, this many "
                         "probed per query) on the same X and report its recall against the exact lists; 0 = skip")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy three times (reference for the profiler's byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU; --gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1807_11824_amd import Tsne, build_P, synth

    dev = torch.device("cuda:0")
    if args.sweep:
        sweep(dev, args.overlap, [int(v) for v in args.sweep_n.split(",")], args.sweep_iters, args.reorder_every,
              args.sweep_approx_tau, args.sweep_recall)
        return
    cache = args.P_cache + ".npz" if args.P_cache else ""
    approx = None
    if cache and os.path.exists(cache):
        from paper_1807_11824_amd import synth as _synth
        cfg = dict(_synth.CONFIGS["cfg5" if args.workload == "cfg5_standin" else args.workload])
        cfg["d_used"] = STANDIN_D if args.workload == "cfg5_standin" else cfg["d"]
        n, k, perp = cfg["n"], cfg["k"], cfg["perplexity"]
        with np.load(cache) as z:
            P = dict(row_ptr=torch.from_numpy(z["row_ptr"]).to(dev), col=torch.from_numpy(z["col"]).to(dev),
                     val=torch.from_numpy(z["val"]).to(dev))
        P["nnz"] = int(P["col"].numel())
        X, t_build = None, None
        nnz = P["nnz"]
    else:
        X, cfg = workload_inputs(args.workload)
        n, k, perp = cfg["n"], cfg["k"], cfg["perplexity"]
        if args.knn_rows > 0:
            Xs = torch.from_numpy(X[:args.knn_rows]).to(dev)
            for rep in range(2):
                torch.cuda.synchronize()
                t0 = time.time()
                Ps = build_P(Xs, perp, k)
                torch.cuda.synchronize()
                print(json.dumps({"knn_rows": int(Xs.shape[0]), "d": int(Xs.shape[1]), "build_P_s": time.time() - t0,
                                  "nnz": Ps["nnz"]}))
            return
        Xd = torch.from_numpy(X).to(dev)
        torch.cuda.synchronize()
        t0 = time.time()
        P = build_P(Xd, perp, k, want_knn=args.approx_tau > 0)
        torch.cuda.synchronize()
        t_build = time.time() - t0
        nnz = P["nnz"]
        if cache:
            np.savez(cache, row_ptr=P["row_ptr"].cpu().numpy(), col=P["col"].cpu().numpy(), val=P["val"].cpu().numpy())
        if args.approx_tau > 0:
            # (not part of the timed steps, which use the exact P: the alternative first phase, timed beside it)
            from paper_1807_11824_amd import build_P_approx
            try:
                t0 = time.time()
                Pa = build_P_approx(Xd, perp, k, args.approx_tau, nlist=0, kmeans_iters=10, want_knn=True)
                torch.cuda.synchronize()
                t_approx = time.time() - t0
                rows = torch.randperm(n, device=dev, generator=torch.Generator(device=dev).manual_seed(0))[:20000]
                hit = (Pa["knn_idx"][rows].long()[:, :, None] == P["knn_idx"][rows].long()[:, None, :]).any(-1)
                approx = {"tau": args.approx_tau, "tau_used": Pa["tau_used"], "nlist": int(round(n ** 0.5)),
                          "kmeans_iters": 10, "second_stage": "flat", "build_P_approx_s": t_approx,
                          "recall_at_k": float(hit.float().mean().item()), "rows_sampled": int(rows.numel()),
                          "nnz": Pa["nnz"]}
                del Pa, hit
            except Exception as e:      # the side measurement must not take the benchmark down with it
                approx = {"tau": args.approx_tau, "error": repr(e)}
        P["knn_idx"] = P["knn_d2"] = None
        del Xd
        torch.cuda.empty_cache()

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    Y0 = synth.y0(n)
    Y0d = torch.from_numpy(Y0).to(dev)
    ts = Tsne(n, overlap=args.overlap, leaf_cap=args.leaf_cap, max_nnz=nnz)
    bits = ts.params.morton_bits
    torch.cuda.synchronize()
    t0 = time.time()
    ts.set_P(P["row_ptr"], P["col"], P["val"])      # renumbers the points and lays the private copy of P out
    torch.cuda.synchronize()
    t_setp = time.time() - t0
    near, far = ts.P_layout()

    # Warm-up: W steps on a scratch copy of Y0, then the optimiser state is reset, so that the timed region is
    # iterations 0 .. K-1 of a real run from Y0 (the state of the embedding decides what an iteration costs).
    if args.warmup:
        scratch = Y0d.clone()
        ts.run(scratch, args.warmup)
        ts.init_state()
        del scratch
    Yd = Y0d.clone()
    torch.cuda.synchronize()
    # every 16th step carries the HIP events of the phase timing (nine event records cost about 30 us)
    every = 16 if args.steps >= 64 else 1
    ts.timing_begin((args.steps + every - 1) // every, every)
    t0 = time.time()
    ts.run(Yd, args.steps)
    torch.cuda.synchronize()
    dt = time.time() - t0
    tm = ts.timing_end()
    status = ts.status()
    if status != 0:
        print(f"bench.py: device status 0x{status:x}", file=sys.stderr)
        sys.exit(1)
    ms_step = dt / args.steps * 1e3
    m_cells = ts.n_cells()

    # A whole run of 1000 iterations from Y0 (no timing events), in chunks of 50 iterations with a host
    # synchronisation between them: what an iteration costs at the start, while the clusters are exaggerated
    # (iteration 100), late (iteration 900), and on average; end to end = build_P + set_P + this run.
    full = None
    if not args.no_full_run:
        ts.init_state()
        Yr = Y0d.clone()
        torch.cuda.synchronize()
        chunk_ms = []
        t_run0 = time.time()
        for c0 in range(0, 1000, 50):
            t0 = time.time()
            ts.run(Yr, 50, iter0=c0)
            torch.cuda.synchronize()
            chunk_ms.append((time.time() - t0) / 50 * 1e3)
        t_run = time.time() - t_run0
        st = ts.status()
        full = {"iterations": 1000, "run_s": t_run, "status": st,
                "iterations_per_s_at_Y0": 1e3 / chunk_ms[0], "iterations_per_s_at_iter_100": 1e3 / chunk_ms[2],
                "iterations_per_s_at_iter_900": 1e3 / chunk_ms[18], "iterations_per_s_whole_run": 1000.0 / t_run,
                "ms_per_iteration_by_chunk_of_50": [round(v, 4) for v in chunk_ms],
                "cells_at_end": ts.n_cells(),
                "end_to_end_s": (t_build + t_setp + t_run) if t_build is not None else None}
        del Yr

    # roofline of the dominant HBM kernels: the attraction streams its private copy of P once (6 bytes per stored
    # entry of the near part, rows padded to 32 entries; 8 bytes per far entry), reads Y once and writes A once.
    # In the timed region it shares the compute units with the walk (overlap), which stretches its launches; the
    # same kernels are timed once more on their own below (30 serial steps) and reported as "standalone".
    radix_passes = (2 * bits + 10) // 11
    sb = step_bytes(n, m_cells, near, far, radix_passes)
    attract_bytes = float(sb["attract"])
    csr_bytes = 8.0 * nnz + 4.0 * (n + 1) + 8.0 * n + 8.0 * n
    phases = dict(tree=tm["tree_ms"], walk=tm["walk_ms"], attract=tm["attract_ms"], update=tm["update_ms"])
    achieved = attract_bytes / (tm["attract_ms"] * 1e-3) / 1e9 if tm["attract_ms"] > 0 else 0.0
    total_bytes = float(sum(sb.values()))
    standalone = None
    if not args.no_standalone:
        solo = Tsne(n, overlap=0, walk_resident=0, leaf_cap=args.leaf_cap, max_nnz=nnz)
        solo.set_P(P["row_ptr"], P["col"], P["val"])
        Ys = Y0d.clone()
        for i in range(5):
            solo.step(Ys, i)
        solo.timing_begin(30)
        for i in range(5, 35):
            solo.step(Ys, i)
        tms = solo.timing_end()
        solo.close()
        del Ys
        solo_achieved = attract_bytes / (tms["attract_ms"] * 1e-3) / 1e9 if tms["attract_ms"] > 0 else 0.0
        standalone = {"ms": tms["attract_ms"], "achieved": solo_achieved, "frac": solo_achieved / HBM_PEAK_GBS,
                      "walk_ms": tms["walk_ms"], "tree_ms": tms["tree_ms"], "update_ms": tms["update_ms"]}
    headline = args.workload == "cfg5"
    out = {
        "metric": "BH t-SNE gradient iterations/sec at N=1.28M" if headline
                  else f"BH t-SNE gradient iterations/sec ({args.workload})",
        "value": args.steps / dt, "unit": "iterations/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: N={n}, D={cfg['d_used']}, k={k}, perplexity={perp}, theta=0.5, "
                               f"P built by tsne_build_P (exact kNN), nnz={nnz}; timed steps = iterations 0..{args.steps - 1} "
                               f"of a run from Y0 (exaggeration 12 for the first 250)"
                               + ("" if args.workload != "cfg5_standin" else
                                  f" -- STAND-IN: X drawn at D'={STANDIN_D}, not the stated D={cfg['d']}"),
                   "n": n, "d": cfg["d_used"], "nnz": nnz, "leaf_cap": args.leaf_cap, "morton_bits": bits,
                   "overlap": args.overlap, "cells": m_cells},
        "phases_ms": phases,
        "build_P_s": t_build,
        "set_P_s": t_setp,
        "step_bytes": {k_: round(v / 1e6, 2) for k_, v in sb.items()},
        "step_bytes_total_GB": total_bytes / 1e9,
        "step_hbm_frac": total_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": {"kernel": "attract_near + attract_far", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     # what rocprofv3's FETCH_SIZE / WRITE_SIZE counted for these kernels on this P, scaled by a
                     # 1 GiB copy (profiles/attract_cfg5_hbm_traffic.md); bytes per step, both kernels
                     "traffic": traffic_from_profile(nnz),
                     "bytes_per_launch": attract_bytes,
                     "bytes_note": "6 B per stored near entry (rows padded to 32) + 8 B per far entry + 24 B per point; "
                                   "a plain CSR of the same P would be csr_bytes",
                     "csr_bytes": csr_bytes,
                     "standalone": standalone},
    }
    if full is not None:
        out["run_1000"] = full
        out["end_to_end_s"] = full["end_to_end_s"]
        out["step_hbm_frac_whole_run"] = total_bytes / (full["run_s"] / 1000.0) / 1e9 / HBM_PEAK_GBS
    if approx is not None:
        out["approx_P"] = approx
        if full is not None and "build_P_approx_s" in approx:
            out["end_to_end_s_approx_P"] = approx["build_P_approx_s"] + t_setp + full["run_s"]
    if not args.no_cpu_baseline:
        P_host = dict(row_ptr=P["row_ptr"].cpu().numpy(), col=P["col"].cpu().numpy(),
                      val=P["val"].cpu().numpy().astype(np.float64))
        out["cpu_baseline"] = cpu_baseline(Y0, P_host, bits, X=X, cfg=cfg, P_gpu_seconds=t_build)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
