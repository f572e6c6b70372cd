"""Throughput of the two-layer network path (config 4 shape) at every K the AdaSync run passes through.

d=3072, 512 hidden units, 10 classes, N=50000 synthetic mixture samples, P=256 virtual workers, m=64,
shifted-exponential delays; K is forced to 8, 16, ..., 256 in turn (the controller is kept from changing
it) and 200 updates are timed at each.  Prints one JSON line per K: microseconds per update,
worker-gradients/s, and the rate of the two bf16 contractions (hidden layer forward, first-layer gradient)
against the 2.5 PFLOP/s dense bf16 MFMA peak.  `--full [J]` runs the whole AdaSync schedule of config 4
instead (J = 20000 updates, K doubling on plateaus) and prints one line for it.  `--replicas R` times K = 8, 16, 32
with R independent replicas in one context (they run beside each other; `us_per_update` is then per update of one
replica, i.e. wall time / (updates x R)).
"""
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_PEAK_TFLOPS = 2500.0


def main(updates=200, ks=(8, 16, 32, 64, 128, 256), replicas=1):
    import torch

    from paper_2003_10579_amd import ssgd, synth

    d, H, C, N, P, m = 3072, 512, 10, 50000, 256, 64
    X, y = synth.mixture_data(N, d, C, seed=0)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ada = dict(mode=1, K0=ks[0], Kmax=256, window=200, rel_tol=-1e9)   # a window never counts as a plateau
    ctx = ssgd.Context("mlp2", Xd, yd, P, ks[0], m, "k_async", ssgd.delay_dist("shifted_exp", 0.5, 1.0), 0.05, seed=0,
                       classes=C, hidden=H, bf16=1, adasync=ada, replicas=replicas)
    R = replicas
    for K in ks:
        ctx.force_K(K)
        ctx.run(updates // 2)          # the first updates after a change still start the previous K's workers
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx.run(updates)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        tr = ctx.trace(0, ctx.updates - updates, updates)
        assert (tr["K"] == K).all()
        flop = R * updates * K * m * 2 * (2 * d * H)      # forward + first-layer gradient contraction
        print(json.dumps({"K": K, "replicas": R, "us_per_update": dt / updates / R * 1e6, "worker_gradients_per_s": R * updates * K / dt,
                          "contraction_tflops": flop / dt / 1e12, "frac_of_bf16_peak": flop / dt / 1e12 / BF16_PEAK_TFLOPS,
                          "mean_loss": float(tr["loss"].mean())}), flush=True)
    ctx.close()


def full_run(J=20000):
    """Config 4 as a whole: AdaSync by plateau doubling (windows of 200 updates, tolerance 0.01) from K = 8 up to 256,
    J updates free-running.  One JSON line: wall time, the updates at which K changed, losses."""
    import torch

    from paper_2003_10579_amd import ssgd, synth

    d, H, C, N, P, m = 3072, 512, 10, 50000, 256, 64
    X, y = synth.mixture_data(N, d, C, seed=0)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ada = dict(mode=1, K0=8, Kmax=256, window=200, rel_tol=0.01)
    ctx = ssgd.Context("mlp2", Xd, yd, P, 8, m, "k_async", ssgd.delay_dist("shifted_exp", 0.5, 1.0), 0.05, seed=0,
                       classes=C, hidden=H, bf16=1, adasync=ada)
    ctx.reserve_trace(J)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ctx.run(J)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tr = ctx.trace()
    K = tr["K"]
    changes = [(int(j), int(K[j])) for j in range(1, J) if K[j] != K[j - 1]]
    grads = int(K.sum())
    print(json.dumps({"workload": "config 4: MLP 3072-512-10, P=256, m=64, AdaSync plateau doubling 8 -> 256, shifted-exp(0.5,1)",
                      "updates": J, "seconds": dt, "worker_gradients": grads, "worker_gradients_per_s": grads / dt,
                      "K_changes_update_newK": changes, "simulated_time": float(tr["t"][-1]),
                      "mean_loss_first_200": float(tr["loss"][:200].mean()), "mean_loss_last_200": float(tr["loss"][-200:].mean()),
                      "full_objective_at_end": ctx.full_loss()}), flush=True)
    ctx.close()


if __name__ == "__main__":
    if len(sys.argv) > 1 and sys.argv[1] == "--full":
        full_run(int(sys.argv[2]) if len(sys.argv) > 2 else 20000)
    elif len(sys.argv) > 2 and sys.argv[1] == "--replicas":
        main(ks=(8, 16, 32), replicas=int(sys.argv[2]))
    else:
        main()
