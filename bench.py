#!/usr/bin/env python3
"""Benchmark of the SuperKMeans hot path on one MI355X.

One *step* is one whole fit (``skm_fit_ex``) of the named workload: rotation GEMM, centroid
initialisation, iteration 1 (full GEMM + argmin), iterations 2..n (initial threshold, partial GEMM +
first test, progressive pruning, argmin, update, d' adjustment), the final two-phase assignment pass
and the un-rotation of the centroids.  Inputs are generated once, seeded, on the GPU and are
resident in HBM when the timed region starts.  The rotation matrix R (a function of d and the seed
only) is made once before the timed region and handed to every fit; the time to make it is reported
separately as ``ms_make_rotation``.

Prints ONE JSON line (see README for the fields).
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

PEAK_FP32_MFMA_TFLOPS = 157.3   # MI355X dense fp32 matrix peak
PEAK_HBM_GBS = 8000.0           # MI355X HBM3E


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="C2", help="workload name in paper_2603_20009_amd.datagen.CONFIGS")
    ap.add_argument("--n", type=int, default=0, help="override the number of points (testing only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=12288)
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "traffic.json"),
                    help="HBM bytes per launch of the dominant kernel from rocprofv3 --pmc runs (optional)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2603_20009_amd import skm, datagen

    cfg = dict(datagen.CONFIGS[args.config])
    n = args.n or cfg["n"]
    d, k, iters = cfg["d"], cfg["k"], cfg["iters"]
    seed = datagen.SEED_FIT
    torch.cuda.set_device(0)
    X = datagen.config_data(args.config, device="cuda", n=n)
    queries = datagen.config_queries(args.config, device="cuda") if cfg.get("etr") else None
    torch.cuda.synchronize()
    t0 = time.time()
    R = skm.make_rotation(d, seed)
    torch.cuda.synchronize()
    ms_make_rotation = (time.time() - t0) * 1e3
    opts = skm.FitOptions(R=R, etr=bool(cfg.get("etr")), queries=queries)

    def step():
        return skm.fit(X, k, iters, seed, opts)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    results = []
    t0 = time.time()
    for _ in range(args.steps):
        results.append(step())
    torch.cuda.synchronize()
    wall = time.time() - t0
    ms_per_step = wall * 1e3 / args.steps
    iters_run = results[-1].iters_run
    value = n * k * d * iters_run / (ms_per_step * 1e-3)

    # ---- per-stage device times (HIP events recorded by the library on its stream), averaged over the steps
    def avg(f):
        return float(np.mean([f(r) for r in results]))

    ds = (d + 15) // 16 * 16
    ms_rot = avg(lambda r: r.timing["ms_rotate"])
    ms_it1_gemm = avg(lambda r: r.trace[0]["ms_gemm"])
    later = lambda r: r.trace[1:]
    ms_filter = avg(lambda r: np.mean([t["ms_gemm"] for t in later(r)]))
    ms_tau = avg(lambda r: np.mean([t["ms_tau"] for t in later(r)]))
    ms_prune = avg(lambda r: np.mean([t["ms_prune"] for t in later(r)]))
    ms_update = avg(lambda r: np.mean([t["ms_update"] for t in r.trace[:r.iters_run]]))
    ms_iter1 = avg(lambda r: r.trace[0]["ms_step"])
    ms_iter_rest = avg(lambda r: np.median([t["ms_step"] for t in r.trace[1:r.iters_run]])) if iters_run > 1 else 0.0
    dprimes = [t["dprime"] for t in results[-1].trace]
    mean_dp = float(np.mean(dprimes[1:])) if len(dprimes) > 1 else 0.0
    surv = [t["survivors"] for t in results[-1].trace[1:]]
    flops_rot = 2.0 * n * d * d
    flops_it1 = 2.0 * n * k * ds
    stages = {
        "rotation_gemm": dict(bound="mfma", ms=ms_rot, achieved=flops_rot / ms_rot / 1e9, unit="TFLOP/s"),
        "iter1_gemm_argmin": dict(bound="mfma", ms=ms_it1_gemm, achieved=flops_it1 / ms_it1_gemm / 1e9, unit="TFLOP/s"),
        "partial_gemm_filter": dict(bound="mfma", ms=ms_filter, achieved=2.0 * n * k * mean_dp / ms_filter / 1e9,
                                    unit="TFLOP/s"),
        "tau_init": dict(bound="hbm", ms=ms_tau, achieved=(n * ds * 4.0 + 24.0 * n) / ms_tau / 1e6, unit="GB/s"),
        "prune": dict(bound="hbm", ms=ms_prune,
                      achieved=(n * (ds - mean_dp) * 4.0 + 16.0 * float(np.mean(surv) if surv else 0)) / ms_prune / 1e6,
                      unit="GB/s"),
        "update": dict(bound="hbm", ms=ms_update, achieved=(n * ds * 4.0 + 8.0 * n + 2.0 * k * ds * 4.0) / ms_update / 1e6,
                       unit="GB/s"),
    }
    for s in stages.values():
        s["frac"] = s["achieved"] / (PEAK_FP32_MFMA_TFLOPS if s["bound"] == "mfma" else PEAK_HBM_GBS)
    # dominant kernel of the fit = the fp32 MFMA GEMM; its longest launch is the rotation (2 n d^2 flop)
    dom = "rotation_gemm" if ms_rot >= ms_it1_gemm else "iter1_gemm_argmin"
    traffic = None
    if os.path.exists(args.traffic_json):
        try:
            traffic = json.load(open(args.traffic_json)).get(args.config, {}).get(dom)
        except Exception:
            traffic = None
    roofline = dict(bound="mfma", kernel=f"skm::gemm_kernel ({dom})", achieved=stages[dom]["achieved"],
                    peak=PEAK_FP32_MFMA_TFLOPS, unit="TFLOP/s", frac=stages[dom]["frac"], traffic=traffic,
                    ms_per_launch=stages[dom]["ms"],
                    flops_per_launch=flops_rot if dom == "rotation_gemm" else flops_it1)

    out = {
        "metric": "point*centroid*dim per second over one SuperKMeans fit (seconds per k-means iteration alongside)",
        "value": value, "unit": "point*centroid*dim/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.config}: {n}x{d} fp32 unit-norm mixture rows ({cfg['components']} components), "
                               f"k={k}, {iters} iterations + final assignment pass", "n": n, "d": d, "k": k,
                   "iters": iters, "iters_run": iters_run},
        "s_per_iteration": {"iteration_1": ms_iter1 * 1e-3, "iterations_2_plus_median": ms_iter_rest * 1e-3,
                            "fit_total_device": avg(lambda r: r.timing["ms_total"]) * 1e-3},
        "ms_make_rotation": ms_make_rotation,
        "ms_before_iteration_1": avg(lambda r: r.timing["ms_init"]),
        "dprime_per_step": dprimes,
        "prune_frac_per_step": [round(t["prune_frac"], 5) for t in results[-1].trace],
        "objective_final": results[-1].trace[-1]["objective"],
        "roofline": roofline,
        "stages": stages,
    }
    if not args.no_cpu_baseline:
        ns = min(n, max(args.cpu_sample, k))
        cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
        out["cpu_baseline"] = cpu_baseline(X[:ns].cpu().numpy(), k, iters, seed, R.cpu().numpy(), cores)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
