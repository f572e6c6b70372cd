"""Rate of the full-objective pass (Eq. (1)) over the d=3072 data set of configs 1, 2 and 4: one JSON line.

  python3 paper_2003_10579_amd/measure_full_loss.py [--passes N]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main(passes=50):
    import torch

    from paper_2003_10579_amd import ssgd, synth

    N, d, C = 50000, 3072, 10
    X, y = synth.mixture_data(N, d, C, seed=0)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ctx = ssgd.Context("softmax", Xd, yd, 8, 2, 32, "k_async", ssgd.delay_dist("shifted_exp", 0.5, 1.0), 0.05, seed=0, classes=C)
    ctx.run(200)
    f = ctx.full_loss()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(passes):
        ctx.full_loss()
    dt = (time.perf_counter() - t0) / passes
    bytes_alg = N * (d + 1) * 4
    print(json.dumps({"workload": f"full objective, softmax d={d}, N={N}", "F_after_200_updates": f, "passes": passes,
                      "us_per_pass_with_host_round_trip": dt * 1e6, "algorithmic_bytes": bytes_alg,
                      "GBps_with_host_round_trip": bytes_alg / dt / 1e9}), flush=True)
    ctx.close()


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--passes", type=int, default=50)
    main(ap.parse_args().passes)
