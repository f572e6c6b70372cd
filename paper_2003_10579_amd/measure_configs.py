"""Throughput of the configurations that bench.py does not time: config 0 (least squares K-sync), config 2
(softmax K-batch-sync, P=64, m=128, K=16, Pareto delays) and config 3 (runtime Monte Carlo, P=128, all K,
10^7 trials per delay distribution), one JSON line each.  Config 3 also reports the largest deviation of the
Exp(1) order-statistic means from their closed form (App. B.1) in standard errors.

  python3 paper_2003_10579_amd/measure_configs.py [--configs 0,2,3] [--mc-trials N]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main(mc_trials=10_000_000, configs=(0, 2, 3)):
    import torch

    from paper_2003_10579_amd import ssgd, synth

    if 0 in configs:
        config0(torch, ssgd, synth)
    if 2 in configs:
        config2(torch, ssgd, synth)
    if 3 in configs:
        config3(ssgd, mc_trials)


def config0(torch, ssgd, synth):
    X, y, _ = synth.lsq_data(4096, 64, 0)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ctx = ssgd.Context("lsq", Xd, yd, 4, 2, 16, "k_sync", ssgd.delay_dist("exp", 1.0), 0.01, seed=0)
    ctx.reserve_trace(1000)
    ctx.run(500)
    t0 = time.perf_counter(); ctx.run(500); dt = time.perf_counter() - t0
    print(json.dumps({"config": 0, "workload": "LSQ K-sync d=64 P=4 m=16 K=2, 500 updates, 1 replica",
                      "us_per_update": dt / 500 * 1e6, "worker_gradients_per_s": 500 * 2 / dt}), flush=True)
    ctx.close()


def config2(torch, ssgd, synth):
    X, y = synth.mixture_data(50000, 3072, 10, seed=0)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    R, J = 40, 200
    ctx = ssgd.Context("softmax", Xd, yd, 64, 16, 128, "k_batch_sync", ssgd.delay_dist("pareto", 2.5, 1.0), 0.05, seed=0,
                       classes=10, replicas=R)
    ctx.reserve_trace(2 * J)
    ctx.run(J)
    t0 = time.perf_counter(); ctx.run(J); dt = time.perf_counter() - t0
    g = R * J * 16 / dt
    print(json.dumps({"config": 2, "workload": f"softmax K-batch-sync d=3072 P=64 m=128 K=16 Pareto(2.5,1), {J} updates, {R} replicas",
                      "us_per_update_per_replica": dt / J * 1e6, "worker_gradients_per_s": g,
                      "algorithmic_GBps": g * 128 * 3073 * 4 / 1e9, "frac_of_8TBps": g * 128 * 3073 * 4 / 8e12}), flush=True)
    ctx.close()


def config3(ssgd, mc_trials):
    P, L = 128, 8
    H = np.cumsum(1.0 / np.arange(1, P + 1))
    for name, spec in (("exp", ("exp", 1.0)), ("shifted_exp", ("shifted_exp", 0.2, 1.0)), ("pareto", ("pareto", 2.5, 1.0))):
        dist = ssgd.delay_dist(*spec)
        ssgd.runtime_mc("k_async", P, 1, P, dist, 2000, L, seed=3)
        t0 = time.perf_counter()
        out = ssgd.runtime_mc("k_async", P, 1, P, dist, mc_trials, L, seed=3)
        dt = time.perf_counter() - t0
        rec = {"config": 3, "distribution": name, "trials": mc_trials, "trials_per_s": mc_trials / dt, "seconds": dt,
               "mean_T1_K64": float(out["mean"][63, 0]), "mean_T8_K64": float(out["mean"][63, 7])}
        if name == "exp":
            exact = np.array([H[P - 1] - (H[P - K - 1] if K < P else 0.0) for K in range(1, P + 1)])
            se = np.sqrt(out["var"] / mc_trials)
            rec["max_abs_dev_in_standard_errors_all_K_all_updates"] = float(np.max(np.abs(out["mean"] - exact[:, None]) / se))
        print(json.dumps(rec), flush=True)

if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="0,2,3")
    ap.add_argument("--mc-trials", type=int, default=10_000_000)
    args = ap.parse_args()
    main(args.mc_trials, tuple(int(c) for c in args.configs.split(",")))
