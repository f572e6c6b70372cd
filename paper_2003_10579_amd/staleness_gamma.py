"""Empirical staleness constants of Sec. 4 on synthetic least squares (the fifth assumption of Sec. 4.1 defines
gamma, the lemma of Sec. 4.2 gives p0): gamma, the smallest constant with
E||grad F(w_j) - grad F(w_tau)||^2 <= gamma E||grad F(w_j)||^2 over the gradients an update uses (tau: the version
its worker read), estimated as the ratio of the two means over a run and its replicas, and p0, the fraction of
fresh gradients.  The full gradients come from `ssgd_full_gradient` after every update.  One JSON line per
(variant, K).

  python3 paper_2003_10579_amd/staleness_gamma.py [--P 8] [--J 300] [--replicas 8] [--dist exp,1.0]
"""
import argparse
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def gamma_estimate(ssgd, Xd, yd, P, K, m, variant, dist_spec, lr, J, replicas, seed=0, keep_params=False, kind="lsq",
                   **model):
    """Runs J updates one at a time; returns the estimate and, on request, every replica's iterates w_0 .. w_J.
    `kind` and `model` (classes=, hidden=, bf16=) choose the model: least squares, softmax regression or the network."""
    ctx = ssgd.Context(kind, Xd, yd, P, K, m, variant, ssgd.delay_dist(*dist_spec), lr, seed=seed, replicas=replicas, **model)
    grads = [[ctx.full_gradient(r).astype(np.float64)] for r in range(replicas)]       # grads[r][j] = grad F(w_j)
    params = [[ctx.params(r)] for r in range(replicas)] if keep_params else None
    for _ in range(J):
        ctx.step()
        for r in range(replicas):
            grads[r].append(ctx.full_gradient(r).astype(np.float64))
            if keep_params:
                params[r].append(ctx.params(r))
    num, den, used, fresh, stale_sum, per_s = 0.0, 0.0, 0, 0, 0, {}
    for r in range(replicas):
        tr = ctx.trace(r)
        for j in range(J):
            gj = grads[r][j]
            den += float(gj @ gj)
            for l in range(int(tr["K"][j])):
                s = int(tr["staleness"][j, l])
                diff = gj - grads[r][j - s]
                v = float(diff @ diff)
                num += v
                used += 1
                fresh += s == 0
                stale_sum += s
                a = per_s.setdefault(s, [0.0, 0])
                a[0] += v
                a[1] += 1
    ctx.close()
    mean_num, mean_den = num / used, den / (replicas * J)
    out = {"variant": variant, "K": K, "P": P, "updates": J, "replicas": replicas,
           "gamma": mean_num / mean_den, "p0": fresh / used, "mean_staleness": stale_sum / used,
           "mean_sq_gradient_difference_by_staleness": {str(s): a[0] / a[1] / mean_den for s, a in sorted(per_s.items())[:12]}}
    return (out, params) if keep_params else out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--P", type=int, default=8)
    ap.add_argument("--J", type=int, default=300)
    ap.add_argument("--replicas", type=int, default=8)
    ap.add_argument("--m", type=int, default=16)
    ap.add_argument("--lr", type=float, default=0.02)
    ap.add_argument("--dist", default="exp,1.0")
    args = ap.parse_args()

    import torch

    from paper_2003_10579_amd import ssgd, synth

    X, y, _ = synth.lsq_data(4096, 256, 0)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    parts = args.dist.split(",")
    spec = (parts[0],) + tuple(float(v) for v in parts[1:])
    for variant in ("k_async", "k_batch_async"):
        for K in [k for k in (1, 2, 4, 8) if k <= args.P]:
            print(json.dumps(gamma_estimate(ssgd, Xd, yd, args.P, K, args.m, variant, spec, args.lr, args.J, args.replicas)),
                  flush=True)


if __name__ == "__main__":
    main()
