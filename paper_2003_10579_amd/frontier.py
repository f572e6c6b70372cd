"""Error-runtime trade-off of the four variants on synthetic least squares (the shape of Fig. 1(b) and of the
error-versus-time figures of Sec. 5; not the paper's CIFAR-10 runs): for every variant and K, R independent replicas
run J updates; reported are the mean simulated time t_J, the mean sub-optimality F(w_J) - F* (the objective over
the whole data set, F* from the normal equations), the mean staleness of the gradients used and the fraction p0 of
fresh ones (p0 of the lemma in Sec. 4.2, used by the error bound of K-async) with the staleness histogram.  One JSON
line per (variant, K).

  python3 paper_2003_10579_amd/frontier.py [--P 8] [--J 600] [--replicas 16] [--dist shifted_exp,1.0,1.0]
"""
import argparse
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

VARIANTS = ("k_sync", "k_batch_sync", "k_async", "k_batch_async")


def frontier(ssgd, Xd, yd, f_star, P, Ks, m, lr, J, replicas, dist_spec, seed=0, variants=VARIANTS):
    """List of records, one per (variant, K)."""
    out = []
    for variant in variants:
        for K in Ks:
            ctx = ssgd.Context("lsq", Xd, yd, P, K, m, variant, ssgd.delay_dist(*dist_spec), lr, seed=seed, replicas=replicas)
            ctx.run(J)
            gaps, times, stale_sum, fresh, used = [], [], 0, 0, 0
            hist = np.zeros(17, dtype=np.int64)         # staleness 0..15, then everything above
            for r in range(replicas):
                gaps.append(ctx.full_loss(r) - f_star)
                tr = ctx.trace(r)
                times.append(float(tr["t"][-1]))
                st = tr["staleness"][tr["sel"] >= 0]
                stale_sum += int(st.sum()); fresh += int((st == 0).sum()); used += int(st.size)
                hist += np.bincount(np.minimum(st, 16), minlength=17)
            ctx.close()
            gaps, times = np.array(gaps), np.array(times)
            out.append({"variant": variant, "K": K, "P": P, "updates": J, "replicas": replicas,
                        "mean_time": float(times.mean()), "time_per_update": float(times.mean() / J),
                        "mean_gap": float(gaps.mean()), "gap_sem": float(gaps.std(ddof=1) / np.sqrt(replicas)) if replicas > 1 else 0.0,
                        "time_by_replica": times.tolist(), "gap_by_replica": gaps.tolist(),
                        "mean_staleness": stale_sum / used, "p0": fresh / used,
                        "staleness_histogram_0_to_15_and_above": (hist / used).round(5).tolist()})
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--P", type=int, default=8)
    ap.add_argument("--J", type=int, default=600)
    ap.add_argument("--replicas", type=int, default=16)
    ap.add_argument("--m", type=int, default=16)
    ap.add_argument("--lr", type=float, default=0.02)
    ap.add_argument("--dist", default="shifted_exp,1.0,1.0")
    args = ap.parse_args()

    import torch

    from paper_2003_10579_amd import ssgd, synth

    X, y, _ = synth.lsq_data(4096, 256, 0)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    X64, y64 = X.astype(np.float64), y.astype(np.float64)
    w_opt = np.linalg.solve(X64.T @ X64, X64.T @ y64)
    f_star = 0.5 * float(np.mean((X64 @ w_opt - y64) ** 2))
    parts = args.dist.split(",")
    spec = (parts[0],) + tuple(float(v) for v in parts[1:])
    Ks = [k for k in (1, 2, 4, 8, 16, 32) if k <= args.P]
    for rec in frontier(ssgd, Xd, yd, f_star, args.P, Ks, args.m, args.lr, args.J, args.replicas, spec):
        print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
