"""Rate of the full-objective pass (Eq. (1)) over the d=3072 data set of configs 1, 2 and 4: one JSON line for the
softmax model and one for the two-layer network of config 4 (hidden 256).

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

    H = 256
    ctx = ssgd.Context("mlp2", Xd, yd, 32, 4, 64, "k_async", ssgd.delay_dist("shifted_exp", 0.5, 1.0), 0.05, seed=0,
                       classes=C, hidden=H, bf16=1)
    ctx.run(20)
    f = ctx.full_loss()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(passes):
        ctx.full_loss()
    dt = (time.perf_counter() - t0) / passes
    flops = 2.0 * N * d * H + 2.0 * N * H * C
    print(json.dumps({"workload": f"full objective, two-layer network d={d}, hidden {H}, N={N}", "F_after_20_updates": f,
                      "passes": passes, "us_per_pass_with_allocation_and_host_round_trips": dt * 1e6,
                      "flop": flops, "TFLOPs": flops / dt / 1e12}), flush=True)
    ctx.close()


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--passes", type=int, default=50)
    main(ap.parse_args().passes)
