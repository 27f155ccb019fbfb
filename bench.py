#!/usr/bin/env python3
"""Benchmark of the SuperKMeans hot path on one MI355X.

One *step* is one whole fit (``skm_fit_ex``) of the headline workload C2 (1M x 1536, k = 1024): rotation GEMM,
centroid initialisation, iteration 1 (full GEMM + argmin), iterations 2..n (initial threshold, partial GEMM + first
test, progressive pruning, argmin, update, d' adjustment), the final two-phase assignment pass and the un-rotation of
the centroids.  Inputs are generated once, seeded, on the GPU and are resident in HBM when the timed region starts.
Every fit makes its own rotation matrix R on the device (fp64 Gram-Schmidt of a seeded Gaussian matrix) inside the
timed region.  The fit's workspace is lent by the caller (a torch tensor sized by ``skm_workspace_bytes``), so a fit
allocates nothing; ``--own-workspace`` lets the library allocate and free it inside every call instead.

Prints ONE JSON line: metric, value (point*centroid*dim per second over whole fits), ms_per_step, the workload in
config, per-iteration seconds, host-clock figures (wall time of a call, wall minus device time), `roofline` for the
dominant kernel (algorithmic flop per launch over its HIP-event time, against the dense fp16 matrix peak divided by
the three products of the split arithmetic), `stages` with the same figures for every kernel family,
`other_workloads` (the rest of the metric's range, k = 4096 ... 32 768: C4, C3, C5, a few timed fits each, same
figures), `hierarchical` (the hierarchical fit of C4 beside the flat one) and `cpu_baseline` (the CPU oracle timed on a bounded sample of the headline workload).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# The GEMM-shaped kernels multiply fp32 operands as scaled (hi, lo) fp16 pairs: three fp16 matrix instructions per
# product (hi*hi' + hi*lo' + lo*hi'), fp32 accumulation.  Their roofline is the dense fp16 matrix peak of MI355X
# divided by those three: the rate at which fp32-class multiply-adds can leave the matrix cores.
PEAK_FP16_MFMA_TFLOPS = 2500.0
SPLIT_PRODUCTS = 3
PEAK_SPLIT_TFLOPS = PEAK_FP16_MFMA_TFLOPS / SPLIT_PRODUCTS
PEAK_HBM_GBS = 8000.0           # MI355X HBM3E
PEAK_FP32_MFMA_TFLOPS = 157.3   # MI355X dense fp32 matrix peak (context: what an fp32 GEMM could reach at most)


def cpu_baseline(X_sample, k, iters, seed, R, cores):
    """The oracle, untuned, on a row sample of the same workload (full k and d)."""
    import numpy as np
    from oracle import oracle
    EPS0 = float(np.float32(2.1))   # the library keeps eps0 in fp32
    oracle.build()
    ns, d = X_sample.shape
    idx = oracle.sample_rows(seed, ns, k)
    t0 = time.time()
    oracle.fit(X_sample, k, iters, seed, oracle.FitParams(eps0=EPS0), R=R, init_idx=idx)
    dt = time.time() - t0
    return dict(value=ns * k * d * iters / dt, unit="point*centroid*dim/s", cores=cores, kind="oracle",
                sample=f"full fit ({iters} iterations + final pass, fp64) on the first {ns} rows of the workload, "
                       f"full k={k} and d={d}; {dt:.1f} s on {cores} threads",
                seconds=dt)


def run_workload(name, steps, warmup, own_workspace, traffic_json, n_override=0):
    """`warmup` untimed and `steps` timed fits of one workload; returns (summary dict, X, results)."""
    import numpy as np
    import torch
    from paper_2603_20009_amd import skm, datagen

    cfg = dict(datagen.CONFIGS[name])
    n = n_override or cfg["n"]
    d, k, iters = cfg["d"], cfg["k"], cfg["iters"]
    seed = datagen.SEED_FIT
    X = datagen.config_data(name, device="cuda", n=n)
    queries = datagen.config_queries(name, device="cuda") if cfg.get("etr") else None
    torch.cuda.synchronize()
    # R = None: made by the fit from the seed
    opts = skm.FitOptions(etr=bool(cfg.get("etr")), queries=queries, own_workspace=own_workspace)

    def step():
        return skm.fit(X, k, iters, seed, opts)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    results = []
    t0 = time.time()
    for _ in range(steps):
        results.append(step())
    torch.cuda.synchronize()
    wall = time.time() - t0
    ms_per_step = wall * 1e3 / steps
    iters_run = results[-1].iters_run
    value = n * k * d * iters_run / (ms_per_step * 1e-3)

    # ---- per-stage device times (HIP events recorded by the library on its stream), averaged over the steps
    def avg(f):
        return float(np.mean([f(r) for r in results]))

    ds = (d + 15) // 16 * 16
    tile_flop = 2.0 * 128 * 128           # MFMA flop per multiplied dimension of one 128 x 128 tile
    ms_rot = avg(lambda r: r.timing["ms_rotate"])
    ms_it1_gemm = avg(lambda r: r.trace[0]["ms_gemm"])
    later = lambda r: r.trace[1:]
    ms_prog = avg(lambda r: np.mean([t["ms_gemm"] for t in later(r)]))
    ms_tau = avg(lambda r: np.mean([t["ms_tau"] for t in later(r)]))
    ms_prune = avg(lambda r: np.mean([t["ms_prune"] for t in later(r)]))
    ms_update = avg(lambda r: np.mean([t["ms_update"] for t in r.trace[:r.iters_run]]))
    ms_iter1 = avg(lambda r: r.trace[0]["ms_step"])
    ms_iter_rest = avg(lambda r: np.median([t["ms_step"] for t in r.trace[1:r.iters_run]])) if iters_run > 1 else 0.0
    last = results[-1]
    dprimes = [t["dprime"] for t in last.trace]
    steps2 = last.trace[1:]
    # algorithmic flop of the progressive kernel per pruned step: the first-test GEMM on d' dims (2 n k d') plus
    # 2 * 64 flop for every (alive pair, trailing block) step that ran inside a dense tile
    flop_alg = float(np.mean([2.0 * n * k * t["dprime"] + 128.0 * t["dense_pair_blocks"] for t in steps2])) if steps2 else 0.0
    flop_exec = float(np.mean([tile_flop * t["dense_dims"] for t in steps2])) if steps2 else 0.0
    total_prog = float(np.sum([t["ms_gemm"] for t in steps2]))
    # algorithmic bytes of the gather kernel per pruned step: a (pair, block) step reads one 256-byte block of the
    # point's row and one of the centroid's block-major copy; every pair is a 16-byte list entry
    prune_bytes = float(np.mean([512.0 * t["gather_pair_blocks"] + 16.0 * t["gather_pairs"] for t in steps2])) if steps2 else 0.0
    # algorithmic bytes of an update: every row once (full), or the rows of the points that changed cluster, twice
    # (joined + left), when the library takes the incremental path (at most one point in eight changed)
    def update_bytes(t, first):
        if not first and 8 * t["changed"] <= n:
            return 2.0 * t["changed"] * ds * 4.0 + 8.0 * n + k * ds * 20.0
        return n * ds * 4.0 + 8.0 * n + 2.0 * k * ds * 4.0
    upd_rows = list(enumerate(last.trace[:last.iters_run]))
    full_upd = [t for i, t in upd_rows if i == 0 or 8 * t["changed"] > n]
    inc_upd = [t for i, t in upd_rows if not (i == 0 or 8 * t["changed"] > n)]
    upd_bytes = float(np.mean([update_bytes(t, i == 0) for i, t in upd_rows]))
    full_bytes = n * ds * 4.0 + 8.0 * n + 2.0 * k * ds * 4.0
    ms_full_upd = float(np.mean([t["ms_update"] for t in full_upd]))
    # threshold pass: every pruned step reads each point once; the first pruned step also writes the split-fp16 copy of the
    # points, its plane of hi halves and the prefix-norm table, and the step that regroups the points writes them again in
    # the new order.  The stage figure is the median step (the steady state); the two special steps are listed beside it.
    tau_ms = sorted(t["ms_tau"] for t in steps2) if steps2 else [0.0]
    ms_tau_med = float(np.median(tau_ms))
    flops_rot = 2.0 * n * d * d
    flops_it1 = 2.0 * n * k * ds
    # one-product (hi * hi') matrix work of the low-precision first filter, in units of one dimension of a 128 x 128 tile
    it1_filtered = last.trace[0]["screen_dims"] > 0
    screen_flop = float(np.mean([tile_flop * t["screen_dims"] for t in steps2])) if steps2 else 0.0
    listed = float(np.mean([t["listed_tiles"] for t in steps2])) if steps2 else 0.0
    n_screened = int(np.sum([t["screen_dims"] > 0 for t in steps2])) if steps2 else 0
    stages = {
        "rotation_gemm": dict(bound="mfma", ms=ms_rot, achieved=flops_rot / ms_rot / 1e9, unit="TFLOP/s"),
        "iter1_gemm_argmin": dict(bound="mfma", ms=ms_it1_gemm, achieved=flops_it1 / ms_it1_gemm / 1e9, unit="TFLOP/s",
                                  filtered=bool(it1_filtered),
                                  one_product_flop=tile_flop * last.trace[0]["screen_dims"],
                                  exact_pairs_per_point=last.trace[0]["gather_pairs"] / n,
                                  note="filtered: one fp16 product per dimension over all pairs keeps, per point, the "
                                       "centroids inside a rigorous error band of the running row minimum; only those "
                                       "pairs get the three-product exact distance (gather kernel), so the matrix work "
                                       "per algorithmic flop is about one third of the unfiltered GEMM's"
                                       if it1_filtered else "unfiltered three-product GEMM with argmin epilogue"),
        "progressive_gemm": dict(bound="mfma", ms=ms_prog, achieved=flop_alg / ms_prog / 1e9, unit="TFLOP/s",
                                 executed=flop_exec / ms_prog / 1e9,
                                 steps_behind_first_filter=n_screened, one_product_flop_per_step=screen_flop,
                                 listed_tiles_per_step=listed),
        "tau_init": dict(bound="hbm", ms=ms_tau_med, achieved=(n * ds * 4.0 + 12.0 * n) / ms_tau_med / 1e6, unit="GB/s",
                         ms_mean=ms_tau, ms_two_largest=tau_ms[-2:],
                         note="median pruned step (reads every point once, writes tau and the incumbent's key); the two "
                              "largest are the first pruned step (also writes the split-fp16 copy of the points, its hi "
                              "plane and the prefix norms) and the step that rewrites the points grouped by cluster"),
        "gather_prune": dict(bound="l2", ms=ms_prune, achieved=(prune_bytes / ms_prune / 1e6) if ms_prune > 0 else None,
                             unit="GB/s", bytes_per_step=prune_bytes,
                             note="requested bytes (512 B per gathered pair-block step + 16 B per pair) over the kernel's "
                                  "time; the blocks of a point and of the centroids are re-read many times and are served "
                                  "by the XCDs' L2 and the Infinity Cache, so this rate is not priced against HBM (no "
                                  "frac); hbm_gbs_rocprof is the kernel's HBM-side rate from the committed counter runs"),
        "update": dict(bound="hbm", ms=ms_full_upd, achieved=full_bytes / ms_full_upd / 1e6, unit="GB/s",
                       full_updates=len(full_upd), incremental_updates=int(last.timing.get("inc_updates", 0)),
                       ms_mean_all=ms_update, achieved_mean_all=upd_bytes / ms_update / 1e6,
                       ms_incremental=[round(t["ms_update"], 4) for t in inc_upd],
                       note="figure of a full update (every row read once: sort by cluster, segmented sums, means); "
                            "incremental updates move only the rows that changed cluster and are latency-bound"),
    }
    for s in stages.values():
        if s["achieved"] is not None and s["bound"] in ("mfma", "hbm"):
            s["frac"] = s["achieved"] / (PEAK_SPLIT_TFLOPS if s["bound"] == "mfma" else PEAK_HBM_GBS)
        if s["achieved"] is not None and s["bound"] == "mfma":
            # the same rate against the chip's fp32 matrix peak (the path an fp32 GEMM would take: 157.3 TFLOP/s)
            s["frac_of_fp32_mfma_peak"] = s["achieved"] / PEAK_FP32_MFMA_TFLOPS
    # dominant kernel of the fit by total time
    totals = {"rotation_gemm": ms_rot, "iter1_gemm_argmin": ms_it1_gemm, "progressive_gemm": total_prog}
    dom = max(totals, key=totals.get)
    traffic = None
    traffic_source = None
    if traffic_json and os.path.exists(traffic_json):
        try:
            per_kernel = json.load(open(traffic_json)).get(name, {})
            traffic = per_kernel.get(dom)
            gp = per_kernel.get("gather_prune")
            if gp and ms_prune > 0:
                # HBM-side bytes per launch (committed rocprofv3 --pmc runs) over this run's time per launch
                stages["gather_prune"]["hbm_bytes_per_launch_rocprof"] = gp["total_bytes"]
                stages["gather_prune"]["hbm_gbs_rocprof"] = gp["total_bytes"] / ms_prune / 1e6
                stages["gather_prune"]["hbm_frac_rocprof"] = gp["total_bytes"] / ms_prune / 1e6 / PEAK_HBM_GBS
            if traffic is not None:
                traffic_source = (f"{os.path.relpath(traffic_json, ROOT)} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of "
                                  f"this command, committed; NOT measured in this run)")
        except Exception:
            traffic = None
    kname = {"rotation_gemm": "skm::gemm_split256_kernel<store>", "iter1_gemm_argmin": "skm::gemm_split256_kernel<argmin>",
             "progressive_gemm": "skm::progressive_kernel"}[dom]
    # traffic: HBM bytes per launch of that kernel (scaled FETCH_SIZE + WRITE_SIZE of the committed counter runs)
    roofline = dict(bound="mfma", kernel=kname, achieved=stages[dom]["achieved"], peak=PEAK_SPLIT_TFLOPS,
                    unit="TFLOP/s", frac=stages[dom]["frac"],
                    frac_of_fp32_mfma_peak=stages[dom]["achieved"] / PEAK_FP32_MFMA_TFLOPS,
                    traffic=None if traffic is None else traffic.get("total_bytes"), traffic_source=traffic_source,
                    traffic_detail=traffic,
                    ms_per_step=stages[dom]["ms"], total_ms_per_fit=totals[dom],
                    flop_per_step={"rotation_gemm": flops_rot, "iter1_gemm_argmin": flops_it1,
                                   "progressive_gemm": flop_alg}[dom],
                    mfma_dtype="f16", mfma_flop_per_algorithmic_flop=SPLIT_PRODUCTS,
                    note="achieved = algorithmic flop (first-test GEMM 2nkd' + 128 per alive pair-block done densely) per "
                         "pruned step / device time of the kernel's launches in that step (HIP events); peak = dense "
                         "fp16 MFMA peak (2500 TFLOP/s) / 3, because every fp32-class product costs three fp16 matrix "
                         "instructions; 'executed' in stages counts every dimension the tiles multiplied")
    if dom == "progressive_gemm":
        roofline["executed"] = stages[dom]["executed"]
        roofline["executed_frac"] = stages[dom]["executed"] / PEAK_SPLIT_TFLOPS
    device_ms = avg(lambda r: r.timing["ms_total"])
    out = {
        "value": value, "unit": "point*centroid*dim/s", "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "config": {"workload": f"{name}: {n}x{d} fp32 unit-norm mixture rows ({cfg['components']} components), "
                               f"k={k}, {iters} iterations + final assignment pass" + (", ETR on 1000 held-out queries" if cfg.get("etr") else ""),
                   "n": n, "d": d, "k": k, "iters": iters, "iters_run": iters_run},
        "s_per_iteration": {"iteration_1": ms_iter1 * 1e-3, "iterations_2_plus_median": ms_iter_rest * 1e-3,
                            "fit_total_device": device_ms * 1e-3},
        "ms_before_iteration_1": avg(lambda r: r.timing["ms_init"]),
        "host": {"ms_call_wall": avg(lambda r: r.timing["ms_host_total"]),
                 "ms_workspace_alloc": avg(lambda r: r.timing["ms_host_alloc"]),
                 "ms_workspace_free": avg(lambda r: r.timing["ms_host_free"]),
                 "ms_wall_minus_device": ms_per_step - device_ms,
                 "workspace": "lent by the caller (a torch tensor; skm_workspace_bytes)" if not own_workspace
                              else "allocated and freed by the library inside every call"},
        "dprime_per_step": dprimes,
        "prune_frac_per_step": [round(t["prune_frac"], 5) for t in last.trace],
        "objective_final": last.trace[-1]["objective"],
        "roofline": roofline,
        "stages": stages,
    }
    if cfg.get("etr"):
        out["recall_per_step"] = [round(t["recall"], 5) for t in last.trace[:iters_run]]
        out["ms_etr_ground_truth"] = avg(lambda r: r.timing["ms_etr_gt"])
    return out, X, results


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="C2", help="headline workload (a name in paper_2603_20009_amd.datagen.CONFIGS)")
    ap.add_argument("--others", default="C4,C3,C5",
                    help="further workloads timed in the same run (comma separated, '' for none): 1 untimed + 3 timed fits each")
    ap.add_argument("--hierarchical", default="C4",
                    help="workload on which the hierarchical fit is timed beside the flat one ('' for none)")
    ap.add_argument("--n", type=int, default=0, help="override the number of points of the headline workload (testing only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--own-workspace", action="store_true",
                    help="let the library allocate and free its workspace inside every call (default: the caller lends it)")
    ap.add_argument("--cpu-sample", type=int, default=24576)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run one 1 GiB device copy first (a kernel of known traffic for scaling rocprofv3 --pmc counters)")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "traffic.json"),
                    help="HBM bytes per launch of the dominant kernel from rocprofv3 --pmc runs (optional)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_20009_amd import skm, datagen

    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)   # 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    head, X, results = run_workload(args.config, args.steps, args.warmup, args.own_workspace, args.traffic_json, args.n)
    out = {
        "metric": "point*centroid*dim per second over one SuperKMeans fit (seconds per k-means iteration alongside)",
        "value": head["value"], "unit": head["unit"],
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "arithmetic": "fp32 in, fp32 accumulation and fp32 out; GEMM-shaped products run on the fp16 matrix cores with "
                      "every operand as a scaled (hi, lo) fp16 pair, 22 significant bits (three MFMAs per product)",
    }
    for key in ("config", "s_per_iteration", "ms_before_iteration_1", "host", "dprime_per_step", "prune_frac_per_step",
                "objective_final", "roofline", "stages"):
        out[key] = head[key]
    cfg = datagen.CONFIGS[args.config]
    if not args.no_cpu_baseline:
        ns = min(X.shape[0], max(args.cpu_sample, cfg["k"]))
        cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
        R = skm.make_rotation(cfg["d"], datagen.SEED_FIT)   # the matrix the fits above used (a function of d and the seed only)
        Xs = X[:ns].cpu().numpy()
        Rn = R.cpu().numpy()
    del X, results
    torch.cuda.empty_cache()
    others = {}
    for name in [s for s in args.others.split(",") if s and s != args.config]:
        o, Xo, ro = run_workload(name, 3, 1, args.own_workspace, args.traffic_json)
        others[name] = o
        del Xo, ro
        torch.cuda.empty_cache()
    out["other_workloads"] = others
    if args.hierarchical and args.hierarchical in datagen.CONFIGS:
        # Hierarchical SuperKMeans (Section 6) on one of the workloads, beside the flat fit of the same k: wall time of
        # whole calls (rotation, meso phase, fine phase, final assignment of all points), 1 untimed + 2 timed
        hc = datagen.CONFIGS[args.hierarchical]
        Xh = datagen.config_data(args.hierarchical, device="cuda")
        torch.cuda.synchronize()
        times = []
        for rep in range(3):
            t0 = time.time()
            hr, sizes, counts = skm.fit_hierarchical(Xh, hc["k"], datagen.SEED_FIT)
            torch.cuda.synchronize()
            times.append((time.time() - t0) * 1e3)
        flat = others.get(args.hierarchical, out if args.hierarchical == args.config else None)
        out["hierarchical"] = {
            "workload": args.hierarchical, "k": hc["k"], "meso_clusters": len(sizes), "meso_iters": 3, "fine_iters": 5,
            "ms_per_fit": float(sum(times[1:]) / 2), "ms_meso_phase": hr.timing["ms_meso"], "ms_fine_phase": hr.timing["ms_fine"],
            "ms_final_assignment": hr.trace[-1]["ms_step"], "final_prune_frac": hr.trace[-1]["prune_frac"],
            "objective": hr.trace[-1]["objective"],
            "objective_over_flat_fit": (hr.trace[-1]["objective"] / flat["objective_final"]) if flat else None,
            "ms_flat_fit": flat["ms_per_step"] if flat else None,
        }
        del Xh, hr
        torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(Xs, cfg["k"], cfg["iters"], datagen.SEED_FIT, Rn, cores)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
