"""Benchmark of the hot path on one MI355X.

Workload: the K-async softmax-regression configuration the metric is quoted on (d=3072, 10 classes,
N=50000 Gaussian-mixture samples, P=8 virtual workers, m=32, K=2, shifted-exponential delays (0.5, 1),
lr=0.05, J=5000 updates), run as R independent replicas, 16 to a launch.  A step is one pass of the whole
hot path: the schedule (delays, K-of-P selection, staleness) and all J updates (gather, gradients at
stale parameters, aggregate, update) of every replica, with the data resident in HBM.
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

HBM_PEAK_GBS = 8000.0


def cpu_baseline(X, y, spec, budget_s=12.0):
    """The oracle, as it stands, on one host core, for a bounded number of updates."""
    import oracle
    tr = oracle.Trainer(oracle.Model("softmax", X, y, classes=10), 8, 2, 32, "k_async", oracle.Dist(*spec), 0.05, seed=0)
    t0 = time.perf_counter()
    done = 0
    while time.perf_counter() - t0 < budget_s and done < 5000:
        tr.run(50)
        done += 50
    dt = time.perf_counter() - t0
    # the oracle's Monte-Carlo estimator, same shape as mc_rate below
    t1 = time.perf_counter()
    oracle.runtime_mc("k_async", 128, 1, 128, oracle.Dist("exp", 1.0), 200, 8, seed=1)
    dt_mc = time.perf_counter() - t1
    return {"value": done * 2 / dt, "unit": "worker-gradients/s", "cores": 1, "kind": "oracle",
            "sample": f"first {done} of 5000 updates of replica 0 ({done * 2} worker-gradients), {dt:.1f} s",
            "mc_trials_per_s": 200 / dt_mc, "mc_sample": f"200 trials (P=128, K=1..128, chains of 8, Exp(1)), {dt_mc:.1f} s"}


KERNEL_SOURCES = ("linear_defer.hip", "linear_tile.hip", "common.hpp")


def kernel_source_hash():
    """sha256 over the sources of the kernels that the timed launches run."""
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2003_10579_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(replicas, updates, grads_per_launch):
    """HBM bytes per launch of the dominant kernel, from the committed counter summary (two rocprofv3 --pmc
    runs of this script, scaled by a copy kernel).  None unless the summary was taken with the same replicas and
    updates and from the kernel sources as they are now (the summary records their hash)."""
    path = os.path.join(ROOT, "profiles", "linear_defer_kernel_config1_hbm_traffic.txt")
    try:
        rec = {}
        with open(path) as f:
            for line in f:
                if line.startswith("bench:"):
                    k, v = line[len("bench:"):].split("=")
                    rec[k.strip()] = v.strip()
        if (int(rec["replicas"]) == replicas and int(rec["updates"]) == updates
                and rec["kernel_source_sha256"] == kernel_source_hash()):
            return (float(rec["fetch_bytes_per_worker_gradient"]) + float(rec["write_bytes_per_worker_gradient"])) * grads_per_launch
    except (OSError, KeyError, ValueError):
        pass
    return None


def config2_rate(ssgd, Xd, yd, replicas=40, updates=200):
    """Config 2 (softmax K-batch-sync, P=64, m=128, K=16, Pareto(2.5, 1) delays) through the same library: worker-gradients
    per second and the fraction of the HBM peak in algorithmic bytes."""
    import torch
    ctx = ssgd.Context("softmax", Xd, yd, 64, 16, 128, "k_batch_sync", ssgd.delay_dist("pareto", 2.5, 1.0), 0.05, seed=0,
                       classes=10, replicas=replicas)
    ctx.reserve_trace(2 * updates)
    ctx.run(updates)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ctx.run(updates)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ctx.close()
    rate = replicas * updates * 16 / dt
    return {"workload": f"config 2: softmax K-batch-sync d=3072 P=64 m=128 K=16 Pareto(2.5,1), {updates} updates, {replicas} replicas",
            "worker_gradients_per_s": rate, "frac_of_hbm_peak": rate * 128 * (3072 + 1) * 4 / 1e9 / HBM_PEAK_GBS}


def config4_rate(ssgd, Xd, yd, updates=4000):
    """Config 4 (two-layer network 3072-512-10, P=256, m=64, K-async, AdaSync by plateau doubling from K=8; bf16 MFMA)
    through the same library: updates and worker-gradients per second of a free run."""
    import torch
    ada = dict(mode=1, K0=8, Kmax=256, window=200, rel_tol=0.01)
    ctx = ssgd.Context("mlp2", Xd, yd, 256, 8, 64, "k_async", ssgd.delay_dist("shifted_exp", 0.5, 1.0), 0.05, seed=0,
                       classes=10, hidden=512, bf16=1, adasync=ada)
    ctx.reserve_trace(updates + 400)
    ctx.run(400)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ctx.run(updates)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    K = ctx.trace(0, 400, updates)["K"]
    ctx.close()
    return {"workload": f"config 4: MLP 3072-512-10 K-async P=256 m=64 AdaSync from K=8, shifted-exp(0.5,1), {updates} updates, 1 replica",
            "us_per_update": dt / updates * 1e6, "worker_gradients_per_s": float(K.sum()) / dt, "K_last": int(K[-1])}


def mc_rate(ssgd):
    """Monte-Carlo runtime estimator (config 3 shape: P=128, every K, K-async chains of 8 updates, Exp(1))."""
    dist = ssgd.delay_dist("exp", 1.0)
    ssgd.runtime_mc("k_async", 128, 1, 128, dist, 2000, 8, seed=1)
    trials = 1000000
    t0 = time.perf_counter()
    ssgd.runtime_mc("k_async", 128, 1, 128, dist, trials, 8, seed=1)
    return trials / (time.perf_counter() - t0)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--replicas", type=int, default=int(os.environ.get("SSGD_BENCH_REPLICAS", "48")))
    ap.add_argument("--updates", type=int, default=5000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); no multi-GPU path exists", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2003_10579_amd import ssgd, synth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    ssgd.lib()
    P, K, m, d, C, N, J, R = 8, 2, 32, 3072, 10, 50000, args.updates, args.replicas
    spec = ("shifted_exp", 0.5, 1.0)
    X, y = synth.mixture_data(N, d, C, seed=0)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()

    def timed(replicas, steps, warmup):
        ctx = ssgd.Context("softmax", Xd, yd, P, K, m, "k_async", ssgd.delay_dist(*spec), 0.05, seed=0, classes=C,
                           replicas=replicas)
        ctx.reserve_trace((steps + warmup) * J)
        for _ in range(warmup):
            ctx.run(J)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        kms, kn = 0.0, 0
        for _ in range(steps):
            ctx.run(J)
            ms, n = ctx.last_kernel_ms()
            kms += ms * n
            kn += n
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        loss = float(ctx.trace(0, ctx.updates - 100, 100)["loss"].mean())
        ctx.close()
        return dt, kms, kn, loss

    dt, kms, kn, loss = timed(R, args.steps, args.warmup)
    grads = R * J * K * args.steps
    value = grads / dt
    b_alg = m * (d + 1) * 4                      # sample rows + labels of one worker-gradient
    per_launch_bytes = grads / kn * b_alg
    achieved = per_launch_bytes / (kms / kn * 1e-3) / 1e9
    dt1, _, _, _ = timed(1, 1, 1)
    out = {
        "metric": "worker-gradients/sec (K-async, d=3072) + % of HBM peak; MC trials/sec",
        "value": value, "unit": "worker-gradients/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config 1: softmax regression K-async, d=3072, 10 classes, N=50000, P=8, m=32, K=2, "
                               f"shifted-exp(0.5,1), lr=0.05, J={J}, {R} independent replicas (16 per launch)",
                   "replicas": R, "updates_per_step": J, "final_loss_replica0": loss,
                   "value_replicas_1": 1 * J * K / dt1},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "linear_defer_kernel<softmax>", "launches": kn, "avg_launch_ms": kms / kn,
                     "algorithmic_bytes_per_launch": per_launch_bytes},
    }
    out["roofline"]["traffic"] = measured_traffic(R, J, grads / kn)
    # what a plain streaming read of the same data set reaches on this device, beside the published peak
    stream_gbs = ssgd.stream_read_rate(Xd, passes=10) / 1e9
    out["roofline"]["stream_read_GBps"] = stream_gbs
    out["roofline"]["frac_of_stream_read"] = achieved / stream_gbs
    if out["roofline"]["traffic"]:
        # the counted HBM-side bytes (sample rows plus the round trip of the parked gradients) against the same ceiling
        out["roofline"]["traffic_GBps"] = out["roofline"]["traffic"] / (kms / kn * 1e-3) / 1e9
        out["roofline"]["traffic_frac_of_stream_read"] = out["roofline"]["traffic_GBps"] / stream_gbs
    out["config"]["config2"] = config2_rate(ssgd, Xd, yd)
    out["config"]["config4"] = config4_rate(ssgd, Xd, yd)
    out["config"]["mc_trials_per_s"] = mc_rate(ssgd)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(X, y, spec)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
