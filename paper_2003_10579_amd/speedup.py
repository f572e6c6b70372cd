"""Runtime speed-ups of Sec. 3 from the Monte-Carlo estimator, one JSON line per P:

  * Theorem 1: E[T_sync] / E[T_async] (K-sync with K = P against K-batch-async with K = 1); for Exp(mu) delays the
    closed form is P (1 + 1/2 + ... + 1/P) ~ P log P.
  * Theorem 2: E[T_K-async] / E[T_K-batch-async] at K = P/2 (first update of a chain against the long-run push rate);
    for Exp(mu): P E[X_{K:P}] / (K E[X]).

  python3 paper_2003_10579_amd/speedup.py [--dist exp,1.0] [--trials 200000]
"""
import argparse
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def speedups(ssgd, spec, Ps=(2, 4, 8, 16, 32, 64, 128, 256), trials=200000, seed=0):
    dist = ssgd.delay_dist(*spec)
    out = []
    for P in Ps:
        K = max(1, P // 2)
        sync = ssgd.runtime_mc("k_sync", P, P, P, dist, trials, 1, seed=seed)["mean"][0, 0]
        # long-run rate of K-batch-async: updates 5..8 of a chain of 8 (past the synchronised start)
        ba1 = ssgd.runtime_mc("k_batch_async", P, 1, 1, dist, trials, 8, seed=seed)["mean"][0, 4:].mean()
        baK = ssgd.runtime_mc("k_batch_async", P, K, K, dist, trials, 8, seed=seed)["mean"][0, 4:].mean()
        kas = ssgd.runtime_mc("k_async", P, K, K, dist, trials, 8, seed=seed)["mean"][0, 4:].mean()
        rec = {"P": P, "sync_over_async": float(sync / ba1), "K": K, "k_async_over_k_batch_async": float(kas / baK)}
        if spec[0] == "exp":
            H = np.cumsum(1.0 / np.arange(1, P + 1))
            rec["theorem1_closed_form"] = float(P * H[P - 1])
            rec["theorem2_closed_form"] = float(P * (H[P - 1] - (H[P - K - 1] if K < P else 0.0)) / K)
        out.append(rec)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dist", default="exp,1.0")
    ap.add_argument("--trials", type=int, default=200000)
    args = ap.parse_args()
    import torch  # noqa: F401  (device context for the library)

    from paper_2003_10579_amd import ssgd

    parts = args.dist.split(",")
    spec = (parts[0],) + tuple(float(v) for v in parts[1:])
    for rec in speedups(ssgd, spec, trials=args.trials):
        print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
