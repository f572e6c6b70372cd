"""The four variants of Sec. 2.2 through the steady-state kernel at the shape of config 1 (softmax regression,
d=3072, 10 classes, N=50000, P=8, m=32, K=2, shifted-exponential delays): microseconds per update and
worker-gradients/s from the kernel launches' HIP events, and the fraction of fresh gradients.  One JSON line per
(variant, replicas).

  python3 paper_2003_10579_amd/measure_variants.py [--updates 3000] [--replicas 16,40]
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--updates", type=int, default=3000)
    ap.add_argument("--replicas", default="16,40")
    args = ap.parse_args()

    import torch

    from paper_2003_10579_amd import ssgd, synth

    P, K, m, d, C, N, J = 8, 2, 32, 3072, 10, 50000, args.updates
    X, y = synth.mixture_data(N, d, C, seed=0)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    for variant in ("k_sync", "k_batch_sync", "k_async", "k_batch_async"):
        for R in [int(v) for v in args.replicas.split(",")]:
            ctx = ssgd.Context("softmax", Xd, yd, P, K, m, variant, ssgd.delay_dist("shifted_exp", 0.5, 1.0), 0.05, seed=0,
                               classes=C, replicas=R)
            ctx.reserve_trace(2 * J + 8)
            ctx.run(J)
            ctx.run(J)
            ms, n = ctx.last_kernel_ms()
            tr = ctx.trace(0)
            st = tr["staleness"][tr["sel"] >= 0]
            print(json.dumps({"variant": variant, "replicas": R, "us_per_update": ms * n / J * 1e3,
                              "worker_gradients_per_s": R * J * K / (ms * n) * 1e3, "fresh_fraction": float((st == 0).mean()),
                              "algorithmic_GBps": R * J * K / (ms * n) * 1e3 * m * (d + 1) * 4 / 1e9}), flush=True)
            ctx.close()


if __name__ == "__main__":
    main()
