"""Parity of the HIP library with the CPU oracle on the same seeded inputs (needs an MI355X).

Bars: delays, sample ids, selections, staleness, ordinals and clock values bit-exact; per-step
averaged gradients within 1e-5 relative (2-norm) in fp32; parameters after J updates within 1e-3
relative.
"""
import math

import numpy as np
import pytest

from paper_2003_10579_amd import synth

pytestmark = pytest.mark.gpu

GRAD_TOL = 1e-5
PARAM_TOL = 1e-3          # the bar the task states for the parameters after J updates
# What fp32 arithmetic supports on the linear models (products and sums of length <= 3072 against fp64;
# the objective is convex, so rounding differences do not grow): asserted wherever the run is fp32.
FP32_PARAM_TOL = 1e-5
FP32_LOSS_RTOL = 2e-5


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


@pytest.fixture(scope="module")
def ssgd():
    from paper_2003_10579_amd import ssgd as s
    s.lib()          # fails loudly if the HIP library is not built
    return s


def rel(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def dist_pair(ssgd, oracle, spec):
    return ssgd.delay_dist(*spec), oracle.Dist(*spec)


def assert_trace_equal(g, o, n=None):
    for k in ("t", "K", "sel", "staleness", "ordinal"):
        a, b = g[k][:n], o[k][:n]
        assert a.shape == b.shape, k
        assert np.array_equal(a, b), (k, np.argwhere(a != b)[:5])


# ------------------------------------------------------------------------------- draws

@pytest.mark.parametrize("spec", [("exp", 1.0), ("exp", 2.5), ("shifted_exp", 0.5, 1.0), ("shifted_exp", 0.2, 1.0),
                                  ("pareto", 2.5, 1.0), ("pareto", 2.0, 1.0), ("pareto", 0.15, 3.0)])
def test_delays_bit_exact(ssgd, oracle, torch_cuda, spec):
    gd, od = dist_pair(ssgd, oracle, spec)
    rng = np.random.default_rng(11)
    bits = rng.integers(0, 2 ** 32, size=400003, dtype=np.uint64).astype(np.uint32)
    bits[:8] = [0, 1, 511, 512, 0xFFFFFFFF, 0xFFFFFE00, 0x80000000, 0x7FFFFFFF]
    got, ref = ssgd.debug_delays(gd, bits), od.from_bits(bits)
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


def test_batch_indices_bit_exact(ssgd, oracle, torch_cuda):
    for (seed, rep, w, o, v, m, N) in [(0, 0, 0, 0, 0, 32, 50000), (7, 3, 255, 2, 19999, 128, 50000),
                                       (2 ** 40 + 5, 63, 17, 0, 4999, 17, 4096), (1, 0, 1, 0, 1, 1, 1),
                                       (9, 1, 2, 3, 4, 64, 2 ** 32 - 1)]:
        got = ssgd.debug_batch(seed, rep, w, o, v, m, N)
        ref = oracle.batch_indices(seed, rep, w, o, v, m, N)
        assert np.array_equal(got, ref)


# ------------------------------------------------------------------------------- schedules

def _tiny(torch, N=64, d=8, seed=0):
    X, y, _ = synth.lsq_data(N, d, seed)
    return X, y, torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()


@pytest.mark.parametrize("variant,P,K,spec", [
    ("k_sync", 4, 2, ("exp", 1.0)), ("k_sync", 100, 37, ("pareto", 2.5, 1.0)), ("k_sync", 256, 256, ("exp", 1.0)),
    ("k_async", 8, 2, ("shifted_exp", 0.5, 1.0)), ("k_async", 1, 1, ("exp", 1.0)), ("k_async", 65, 9, ("pareto", 2.5, 1.0)),
    ("k_async", 256, 8, ("shifted_exp", 0.5, 1.0)), ("k_async", 256, 255, ("exp", 3.0)),
    ("k_async", 16, 5, ("exp", 1.0)), ("k_async", 64, 16, ("pareto", 2.5, 1.0)), ("k_async", 200, 40, ("shifted_exp", 0.2, 1.0)),
    ("k_async", 17, 16, ("exp", 1.0)),
    ("k_batch_sync", 64, 16, ("pareto", 2.5, 1.0)), ("k_batch_sync", 3, 7, ("exp", 1.0)), ("k_batch_sync", 130, 1, ("exp", 1.0)),
])
def test_schedule_bit_exact(ssgd, oracle, torch_cuda, variant, P, K, spec):
    """Delays, K-of-P selection, staleness, ordinals, clock: GPU trace == oracle trace."""
    X, y, Xd, yd = _tiny(torch_cuda)
    gd, od = dist_pair(ssgd, oracle, spec)
    J = 150
    ctx = ssgd.Context("lsq", Xd, yd, P, K, 1, variant, gd, 0.0, seed=5)
    ctx.run(60)
    ctx.run(J - 60)          # a second call continues the same event process
    tr = oracle.Trainer(oracle.Model("lsq", X, y), P, K, 1, variant, od, 0.0, seed=5)
    tr.run(J)
    assert ctx.updates == J
    assert_trace_equal(ctx.trace(), tr.trace())
    ctx.close()


def test_schedule_table_ties_and_dead_worker(ssgd, oracle, torch_cuda):
    X, y, Xd, yd = _tiny(torch_cuda)
    rng = np.random.default_rng(3)
    for variant, P, K in [("k_sync", 4, 2), ("k_async", 4, 3), ("k_batch_sync", 3, 4), ("k_async", 5, 1)]:
        R = K + 1 if "batch" in variant else 1
        table = np.float32(rng.integers(1, 4, size=(41 * P * R)) * 0.5).reshape(41, P, R)
        if P - 1 >= K:
            table[:, P - 1, :] = np.inf
        gd, od = dist_pair(ssgd, oracle, ("table", table.ravel()))
        ctx = ssgd.Context("lsq", Xd, yd, P, K, 2, variant, gd, 0.01, seed=1)
        ctx.run(40)
        tr = oracle.Trainer(oracle.Model("lsq", X, y), P, K, 2, variant, od, 0.01, seed=1)
        tr.run(40)
        assert_trace_equal(ctx.trace(), tr.trace())
        ctx.close()


# ------------------------------------------------------------------------------- training parity

def _run_pair(ssgd, oracle, torch, kind, X, y, P, K, m, variant, spec, lr, J, seed=0, classes=1, check_steps=40):
    """Per-step averaged gradients (teacher-forced from the oracle's iterate where the variant keeps no
    in-flight gradients, i.e. the sync variants; free-running otherwise), then a free run of J updates
    for the trace and the final parameters.  Single updates go through the same kernels as whole runs:
    the steady-state kernel wherever the shape allows it (from update 1 on for K-async)."""
    gd, od = dist_pair(ssgd, oracle, spec)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    mk_ctx = lambda: ssgd.Context(kind, Xd, yd, P, K, m, variant, gd, lr, seed=seed, classes=classes)
    mk_orc = lambda: oracle.Trainer(oracle.Model(kind, X, y, classes=classes), P, K, m, variant, od, lr, seed=seed)
    ctx, tr = mk_ctx(), mk_orc()
    agg = torch.zeros(ctx.nw, dtype=torch.float32, device="cuda")
    forced = variant in ("k_sync", "k_batch_sync")
    worst = 0.0
    for j in range(min(check_steps, J)):
        if forced:
            ctx.set_params(tr.params())
        ctx.step(agg)
        worst = max(worst, rel(agg.cpu().numpy(), tr.step()))
    if forced:
        ctx.close()
        ctx, tr = mk_ctx(), mk_orc()
        ctx.run(J)
        tr.run(J)
    elif J > check_steps:
        ctx.run(J - check_steps)
        tr.run(J - check_steps)
    gt, ot = ctx.trace(), tr.trace()
    assert_trace_equal(gt, ot)
    pr = rel(ctx.params(), tr.params())
    print(f"worst per-step gradient error {worst:.3e}, parameter error after {J} updates {pr:.3e}")
    assert worst <= GRAD_TOL, worst
    assert np.allclose(gt["loss"], ot["loss"], rtol=FP32_LOSS_RTOL, atol=1e-6)
    assert pr <= FP32_PARAM_TOL, pr
    ctx.close()
    return worst, pr


def test_config0_lsq_ksync_full(ssgd, oracle, torch_cuda):
    """d=64, N=4096, P=4, m=16, K=2, Exp(1), lr=0.01, J=500, seed 0."""
    X, y, _ = synth.lsq_data(4096, 64, 0)
    _run_pair(ssgd, oracle, torch_cuda, "lsq", X, y, 4, 2, 16, "k_sync", ("exp", 1.0), 0.01, 500, check_steps=500)


@pytest.mark.parametrize("variant,P,K,m,d,classes,spec", [
    ("k_async", 8, 2, 32, 320, 10, ("shifted_exp", 0.5, 1.0)),      # two records per tile, two slices
    ("k_async", 5, 3, 5, 100, 3, ("exp", 1.0)),                      # m not a multiple of 4, ragged last slice
    ("k_async", 3, 1, 100, 70, 4, ("pareto", 2.5, 1.0)),             # m > 64 (two sub-tiles), d % 4 != 0
    ("k_sync", 6, 4, 16, 520, 10, ("exp", 1.0)),                     # three slices, last one ragged
    ("k_batch_sync", 6, 9, 20, 256, 16, ("pareto", 2.5, 1.0)),       # K > P, 16 classes, exactly one slice
    ("k_sync", 2, 2, 64, 64, 2, ("exp", 1.0)),                       # one full tile per record
    ("k_batch_sync", 4, 3, 128, 300, 10, ("shifted_exp", 0.5, 1.0)),
])
def test_softmax_parity_small(ssgd, oracle, torch_cuda, variant, P, K, m, d, classes, spec):
    X, y = synth.mixture_data(1500, d, classes, seed=1)
    _run_pair(ssgd, oracle, torch_cuda, "softmax", X, y, P, K, m, variant, spec, 0.05, 120, seed=3, classes=classes)


@pytest.mark.parametrize("variant,P,K,m,d", [("k_async", 4, 2, 16, 64), ("k_async", 7, 2, 9, 33), ("k_batch_sync", 3, 5, 70, 130)])
def test_lsq_parity_small(ssgd, oracle, torch_cuda, variant, P, K, m, d):
    X, y, _ = synth.lsq_data(900, d, 2)
    _run_pair(ssgd, oracle, torch_cuda, "lsq", X, y, P, K, m, variant, ("exp", 1.0), 0.01, 150, seed=4)


@pytest.mark.parametrize("kind,variant,P,K,m,N,d,classes", [
    ("lsq", "k_sync", 1, 1, 1, 50, 4, 1),             # serial SGD on single samples
    ("softmax", "k_async", 1, 1, 3, 40, 8, 2),        # one worker: never stale
    ("lsq", "k_async", 3, 2, 4, 1, 12, 1),            # a data set of one sample: every index is 0
    ("lsq", "k_sync", 256, 256, 1, 300, 16, 1),       # the largest number of workers, all of them waited for
    ("softmax", "k_batch_sync", 2, 256, 1, 64, 8, 3), # ordinals up to 255 on two workers
    ("softmax", "k_async", 256, 1, 2, 500, 260, 10),  # fully asynchronous, staleness in the hundreds
])
def test_degenerate_and_extreme_shapes(ssgd, oracle, torch_cuda, kind, variant, P, K, m, N, d, classes):
    if kind == "lsq":
        X, y, _ = synth.lsq_data(N, d, 9)
    else:
        X, y = synth.mixture_data(N, d, classes, seed=9)
    _run_pair(ssgd, oracle, torch_cuda, kind, X, y, P, K, m, variant, ("exp", 1.0), 0.01, 30, seed=2, classes=classes,
              check_steps=30)


def test_run_of_zero_updates_changes_nothing(ssgd, torch_cuda):
    torch = torch_cuda
    X, y, _ = synth.lsq_data(200, 16, 5)
    ctx = ssgd.Context("lsq", torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda(), 4, 2, 8, "k_async",
                       ssgd.delay_dist("exp", 1.0), 0.01, seed=1)
    ctx.run(0)
    assert ctx.updates == 0 and not ctx.params().any()
    ctx.run(5)
    before = ctx.params().copy()
    ctx.run(0)
    assert ctx.updates == 5 and np.array_equal(ctx.params(), before)
    ctx.close()


def test_replicas_are_independent_runs(ssgd, oracle, torch_cuda):
    """Replica r of one context == a single-replica oracle run keyed by r; 19 replicas span three
    launch groups of eight."""
    torch = torch_cuda
    X, y = synth.mixture_data(1200, 320, 10, seed=2)
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.5, 1.0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ctx = ssgd.Context("softmax", Xd, yd, 8, 2, 32, "k_async", gd, 0.05, seed=6, classes=10, replicas=19)
    ctx.run(80)
    for r in (0, 1, 7, 8, 18):
        tr = oracle.Trainer(oracle.Model("softmax", X, y, classes=10), 8, 2, 32, "k_async", od, 0.05, seed=6, replica=r)
        tr.run(80)
        assert_trace_equal(ctx.trace(r), tr.trace())
        assert rel(ctx.params(r), tr.params()) <= FP32_PARAM_TOL
        assert np.allclose(ctx.trace(r)["loss"], tr.trace()["loss"], rtol=FP32_LOSS_RTOL, atol=1e-6)
    assert not np.array_equal(ctx.params(0), ctx.params(1))
    ctx.close()


def test_set_params_teacher_forcing(ssgd, oracle, torch_cuda):
    """Per-step gradient parity from the oracle's own iterate (sync variant: no parked state)."""
    torch = torch_cuda
    X, y = synth.mixture_data(1000, 200, 10, seed=5)
    gd, od = dist_pair(ssgd, oracle, ("exp", 1.0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ctx = ssgd.Context("softmax", Xd, yd, 6, 3, 24, "k_sync", gd, 0.2, seed=8, classes=10)
    tr = oracle.Trainer(oracle.Model("softmax", X, y, classes=10), 6, 3, 24, "k_sync", od, 0.2, seed=8)
    agg = torch.zeros(ctx.nw, device="cuda")
    for j in range(60):
        ctx.set_params(tr.params())
        ctx.step(agg)
        g = tr.step()
        assert rel(agg.cpu().numpy(), g) <= GRAD_TOL
    ctx.close()


def test_adasync_plateau_mode(ssgd, oracle, torch_cuda):
    torch = torch_cuda
    X, y = synth.mixture_data(1500, 128, 10, seed=7)
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.5, 1.0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ada = dict(mode=1, K0=1, Kmax=16, window=25, rel_tol=0.01)
    ctx = ssgd.Context("softmax", Xd, yd, 16, 1, 8, "k_async", gd, 0.05, seed=2, classes=10, adasync=ada)
    tr = oracle.Trainer(oracle.Model("softmax", X, y, classes=10), 16, 1, 8, "k_async", od, 0.05, seed=2, adasync=ada)
    ctx.run(130)
    ctx.run(270)
    tr.run(400)
    g, o = ctx.trace(), tr.trace()
    assert o["K"][-1] > 1
    # the doubling decision compares two fp32-derived means; both sides agree unless a window mean
    # sits within rounding of the threshold, so compare exactly and report the first difference
    assert np.array_equal(g["K"], o["K"]), np.argwhere(g["K"] != o["K"])[:3]
    assert_trace_equal(g, o)
    assert rel(ctx.params(), tr.params()) <= FP32_PARAM_TOL
    ctx.close()


@pytest.mark.parametrize("mode,variant", [(2, "k_async"), (3, "k_sync")])
def test_adasync_paper_rules(ssgd, oracle, torch_cuda, mode, variant):
    torch = torch_cuda
    X, y, _ = synth.lsq_data(512, 16, 3)
    gd, od = dist_pair(ssgd, oracle, ("exp", 1.0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ada = dict(mode=mode, K0=2, Kmax=16, interval_t=6.0)
    ctx = ssgd.Context("lsq", Xd, yd, 16, 2, 4, variant, gd, 0.03, seed=2, adasync=ada)
    tr = oracle.Trainer(oracle.Model("lsq", X, y), 16, 2, 4, variant, od, 0.03, seed=2, adasync=ada)
    ctx.run(300)
    tr.run(300)
    g, o = ctx.trace(), tr.trace()
    assert o["K"][-1] > 2
    assert np.array_equal(g["K"], o["K"])
    assert_trace_equal(g, o)
    ctx.close()


# ------------------------------------------------------------------------------- full-size configurations

@pytest.fixture(scope="module")
def mixture_full(torch_cuda):
    X, y = synth.mixture_data(50000, 3072, 10, seed=0)
    return X, y, torch_cuda.from_numpy(X).cuda(), torch_cuda.from_numpy(y).cuda()


@pytest.fixture(scope="module")
def config2_oracle_run(oracle, mixture_full):
    """The oracle's whole run of config 2 (2000 iterations of 16 x 128 rows at d=3072 take it minutes on one core),
    started in a thread of its own the first time a full-size test asks for the data, collected by the config 2
    test at the end of the module.  The oracle keeps no state outside a Trainer and its calls release the
    interpreter lock."""
    import threading
    from concurrent.futures import ThreadPoolExecutor
    X, y, _, _ = mixture_full

    def run():
        tr = oracle.Trainer(oracle.Model("softmax", X, y, classes=10), 64, 16, 128, "k_batch_sync",
                            oracle.Dist("pareto", 2.5, 1.0), 0.05, seed=0)
        for _ in range(20):
            if stop.is_set():     # the module's tests are over (one of them failed): do not hold up the exit
                break
            tr.run(100)
        return tr

    stop = threading.Event()
    pool = ThreadPoolExecutor(max_workers=1)
    fut = pool.submit(run)
    yield fut
    stop.set()
    pool.shutdown(wait=False, cancel_futures=True)


def test_config1_softmax_kasync_full_size(ssgd, oracle, torch_cuda, mixture_full, config2_oracle_run):
    """d=3072, N=50000, 10 classes, P=8, m=32, K=2, shifted-Exp(0.5, 1), lr=0.05, J=5000, in the benchmark's launch
    configuration (many replicas in one launch).  The oracle follows replica 0 through all 5000 updates (30 of them
    as single steps with the averaged gradient compared, from update 1 on through the steady-state kernel) and
    replica 37 for the first 600; schedule, loss trace and the parameters at J against it."""
    torch = torch_cuda
    X, y, Xd, yd = mixture_full
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.5, 1.0))
    R, J = 40, 5000
    ctx = ssgd.Context("softmax", Xd, yd, 8, 2, 32, "k_async", gd, 0.05, seed=0, classes=10, replicas=R)
    agg = torch.zeros(ctx.nw, device="cuda")
    tr0 = oracle.Trainer(oracle.Model("softmax", X, y, classes=10), 8, 2, 32, "k_async", od, 0.05, seed=0, replica=0)
    worst = 0.0
    for j in range(30):
        ctx.step(agg)
        worst = max(worst, rel(agg.cpu().numpy(), tr0.step()))
    assert worst <= GRAD_TOL, worst
    ctx.run(570)
    tr37 = oracle.Trainer(oracle.Model("softmax", X, y, classes=10), 8, 2, 32, "k_async", od, 0.05, seed=0, replica=37)
    tr37.run(600)
    assert_trace_equal(ctx.trace(37), tr37.trace())
    assert rel(ctx.params(37), tr37.params()) <= FP32_PARAM_TOL
    assert np.allclose(ctx.trace(37)["loss"], tr37.trace()["loss"], rtol=FP32_LOSS_RTOL, atol=1e-6)
    ctx.run(J - 600)
    tr0.run(J - 30)
    assert ctx.updates == J and tr0.updates == J
    assert_trace_equal(ctx.trace(0), tr0.trace())
    pr = rel(ctx.params(0), tr0.params())
    print(f"config 1: worst per-step gradient error {worst:.3e}, parameter error after {J} updates {pr:.3e}")
    assert pr <= FP32_PARAM_TOL, pr
    assert np.allclose(ctx.trace(0)["loss"], tr0.trace()["loss"], rtol=FP32_LOSS_RTOL, atol=1e-6)
    # schedule of the whole run of another replica against an oracle that skips the gradients (tiny stand-in model)
    Xs, ys, _ = synth.lsq_data(16, 2, 0)
    sched = oracle.Trainer(oracle.Model("lsq", Xs, ys), 8, 2, 1, "k_async", od, 0.0, seed=0, replica=37)
    sched.run(J)
    assert_trace_equal(ctx.trace(37), sched.trace())
    w = ctx.params(37)
    assert np.all(np.isfinite(w)) and ctx.trace(37)["loss"][-200:].mean() < ctx.trace(37)["loss"][:50].mean()
    ctx.close()


@pytest.mark.parametrize("variant", ["k_sync", "k_batch_sync"])
def test_steady_state_kernel_single_steps_at_the_benchmark_launch_shape(ssgd, oracle, torch_cuda, variant):
    """Eq. (2) at the launch shape of config 1 (d=3072: twelve column slices, 40 replicas in one launch, P=8, m=32,
    K=2): every single step of replica 0 goes through the steady-state kernel, teacher-forced from the oracle's
    iterate, the averaged gradient within 1e-5."""
    torch = torch_cuda
    X, y = synth.mixture_data(3000, 3072, 10, seed=3)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.5, 1.0))
    ctx = ssgd.Context("softmax", Xd, yd, 8, 2, 32, variant, gd, 0.05, seed=4, classes=10, replicas=40)
    tr = oracle.Trainer(oracle.Model("softmax", X, y, classes=10), 8, 2, 32, variant, od, 0.05, seed=4)
    agg = torch.zeros(ctx.nw, device="cuda")
    worst = 0.0
    for j in range(40):
        ctx.set_params(tr.params())
        ctx.step(agg)
        worst = max(worst, rel(agg.cpu().numpy(), tr.step()))
    print(f"{variant}: worst per-step gradient error {worst:.3e}")
    assert worst <= GRAD_TOL, worst
    assert_trace_equal(ctx.trace(), tr.trace())
    ctx.close()


def test_general_kernel_single_steps(ssgd, oracle, torch_cuda, monkeypatch):
    """The general kernel, forced for a shape the steady-state kernel would take: same bars."""
    monkeypatch.setenv("SSGD_KERNEL", "general")
    X, y = synth.mixture_data(1500, 320, 10, seed=1)
    _run_pair(ssgd, oracle, torch_cuda, "softmax", X, y, 8, 2, 32, "k_async", ("shifted_exp", 0.5, 1.0), 0.05, 120, seed=3,
              classes=10)


# ------------------------------------------------------------------------------- Monte Carlo

@pytest.mark.parametrize("variant,P,Kmax,spec", [
    ("k_async", 128, 128, ("exp", 1.0)), ("k_async", 128, 128, ("shifted_exp", 0.2, 1.0)),
    ("k_async", 128, 128, ("pareto", 2.5, 1.0)), ("k_async", 5, 5, ("exp", 1.0)), ("k_async", 200, 200, ("pareto", 2.5, 1.0)),
    ("k_sync", 128, 128, ("pareto", 2.5, 1.0)), ("k_sync", 64, 64, ("exp", 2.0)),
    ("k_batch_sync", 6, 9, ("exp", 1.5)), ("k_batch_sync", 70, 20, ("shifted_exp", 0.2, 1.0)),
    ("k_batch_async", 128, 128, ("pareto", 2.0, 1.0)), ("k_batch_async", 6, 9, ("exp", 1.5)),
    ("k_batch_async", 200, 40, ("shifted_exp", 1.0, 1.0)),
])
def test_mc_trials_bit_exact(ssgd, oracle, torch_cuda, variant, P, Kmax, spec):
    gd, od = dist_pair(ssgd, oracle, spec)
    L = 8 if Kmax * 8 * 16 <= 65536 else 4
    trials = 300 if P < 200 else 100
    g = ssgd.runtime_mc(variant, P, 1, Kmax, gd, trials, L, seed=9, trial0=5, per_trial=True)
    o = oracle.runtime_mc(variant, P, 1, Kmax, od, trials, L, seed=9, trial0=5, per_trial=True)
    assert np.array_equal(g["per_trial"], o["per_trial"])
    assert np.allclose(g["sum"], o["sum"], rtol=1e-12)
    assert np.allclose(g["sumsq"], o["sumsq"], rtol=1e-12)
    assert np.allclose(g["mean"], o["mean"], rtol=1e-12) and np.allclose(g["var"], o["var"], rtol=1e-9)


@pytest.mark.parametrize("variant", ["k_async", "k_sync", "k_batch_async"])
def test_mc_ten_thousand_trials_bit_exact(ssgd, oracle, torch_cuda, variant):
    """The first 10^4 trials of one shape (P=16, every K, chains of 4 updates, shifted-exponential delays), trial by
    trial and in the sums."""
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.2, 1.0))
    g = ssgd.runtime_mc(variant, 16, 1, 16, gd, 10000, 4, seed=3, per_trial=True)
    o = oracle.runtime_mc(variant, 16, 1, 16, od, 10000, 4, seed=3, per_trial=True)
    assert np.array_equal(g["per_trial"], o["per_trial"])
    assert np.allclose(g["sum"], o["sum"], rtol=1e-12) and np.allclose(g["sumsq"], o["sumsq"], rtol=1e-12)


def test_mc_closed_forms_at_scale(ssgd, torch_cuda):
    """2e5 trials, P=128, all K: Exp(1) order statistics (App. B.1) for every update of the K-async chain
    (App. B.3); shifted exponential first update = shift + harmonic form; K-async <= K-sync afterwards."""
    P, n, L = 128, 200000, 8
    Ks = np.arange(1, P + 1)
    H = np.array([sum(1.0 / i for i in range(P - K + 1, P + 1)) for K in Ks])
    V = np.array([sum(1.0 / i ** 2 for i in range(P - K + 1, P + 1)) for K in Ks])
    r = ssgd.runtime_mc("k_async", P, 1, P, ssgd.delay_dist("exp", 1.0), n, L, seed=1)
    for l in range(L):
        assert np.all(np.abs(r["mean"][:, l] - H) <= 5 * np.sqrt(V / n))
        assert np.all(np.abs(r["var"][:, l] / V - 1) < 0.05)
    s = ssgd.runtime_mc("k_async", P, 1, P, ssgd.delay_dist("shifted_exp", 0.2, 1.0), n, L, seed=2)
    assert np.all(np.abs(s["mean"][:, 0] - (0.2 + H)) <= 5 * np.sqrt(V / n))
    assert np.all(s["mean"][:, 1:] <= (0.2 + H)[:, None] + 5 * np.sqrt(s["var"][:, 1:] / n))


def test_mc_kbatch_async_closed_form_at_scale(ssgd, torch_cuda):
    """Lemma 5 / Theorem 2 at P=128: with Exp(mu) delays every inter-update time of K-batch-async is Erlang(K, P mu),
    mean K/(P mu), variance K/(P mu)^2, for all K and every update of the chain; 2e5 trials."""
    P, n, L, mu = 128, 200000, 8, 2.0
    Ks = np.arange(1, P + 1)
    r = ssgd.runtime_mc("k_batch_async", P, 1, P, ssgd.delay_dist("exp", mu), n, L, seed=4)
    mean, var = Ks / (P * mu), Ks / (P * mu) ** 2
    for l in range(L):
        assert np.all(np.abs(r["mean"][:, l] - mean) <= 5 * np.sqrt(var / n))
        assert np.all(np.abs(r["var"][:, l] / var - 1) < 0.05)


# ---------------------------------------------------------------------------------------------
# Two-layer ReLU network (bf16 operands, fp32 accumulation).  Tolerances: the oracle accumulates the
# bf16 products in fp64, the MFMA units in fp32 (relative 1e-6 per dot product of length d); what makes
# the difference visible are decisions taken on those sums -- a hidden unit whose pre-activation is
# within that error of zero switches its ReLU mask, and a delta1 value within it of a bf16 rounding
# boundary moves by one bf16 ulp (2^-8 relative) -- each a rare, isolated change of one entry.
MLP_GRAD_TOL = 3e-4     # observed: 6e-7 ... 9e-5, and 1.9e-4 for the mean of 256 gradients at full size (more cancellation)
MLP_PARAM_TOL = 2e-3


def _mlp_pair(ssgd, oracle, torch, X, y, P, K, m, variant, spec, lr, classes, hidden, seed=0, adasync=None):
    gd, od = dist_pair(ssgd, oracle, spec)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ctx = ssgd.Context("mlp2", Xd, yd, P, K, m, variant, gd, lr, seed=seed, classes=classes, hidden=hidden, bf16=1,
                       adasync=adasync)
    tr = oracle.Trainer(oracle.Model("mlp2", X, y, classes=classes, hidden=hidden, bf16=1), P, K, m, variant, od, lr,
                        seed=seed, adasync=adasync)
    return ctx, tr


def test_mlp_initial_parameters_bit_exact(ssgd, oracle, torch_cuda):
    X, y = synth.mixture_data(600, 256, 5, seed=2)
    ctx, tr = _mlp_pair(ssgd, oracle, torch_cuda, X, y, 4, 2, 16, "k_sync", ("exp", 1.0), 0.05, 5, 128, seed=11)
    assert np.array_equal(ctx.params(), tr.params())
    ctx.close()


@pytest.mark.parametrize("variant,P,K,m,d,classes,hidden", [
    ("k_sync", 4, 2, 64, 256, 10, 128),
    ("k_sync", 6, 3, 20, 128, 3, 256),        # m < 64: zero rows in every block
    ("k_async", 6, 2, 32, 384, 10, 128),
    ("k_batch_sync", 3, 5, 16, 128, 4, 128),  # a worker contributes more than once (K > P)
    ("k_sync", 80, 64, 4, 128, 5, 128),       # 64 slots per update: the gradient contraction is split into four shares
    ("k_async", 100, 90, 3, 256, 4, 128),     # five shares of 18 slots; ranked selection in the schedule
    ("k_batch_async", 6, 3, 16, 256, 5, 128),  # mini-batches started and consumed inside one update
    ("k_batch_async", 3, 5, 64, 128, 4, 128),  # K > P: a worker pushes several times per update
    ("k_batch_async", 40, 70, 4, 128, 3, 128), # 109 records at version 0, split gradient contraction
    ("k_batch_async", 5, 1, 64, 128, 16, 128), # K = 1: fully asynchronous SGD
    ("k_sync", 80, 64, 4, 256, 5, 512),        # 512 hidden units: four rows of 128 x 128 tiles in the split contraction
    ("k_async", 130, 128, 2, 384, 10, 512),    # eight shares of 16 slots, four rows and three columns of tiles
])
def test_mlp_gradients_teacher_forced(ssgd, oracle, torch_cuda, variant, P, K, m, d, classes, hidden):
    """Every update's averaged gradient against the oracle's.  K-sync is teacher-forced (the oracle's iterate is
    loaded before each step); the asynchronous variants run free, their in-flight factors depend on earlier
    iterates."""
    torch = torch_cuda
    X, y = synth.mixture_data(2000, d, classes, seed=4)
    ctx, tr = _mlp_pair(ssgd, oracle, torch, X, y, P, K, m, variant, ("shifted_exp", 0.5, 1.0), 0.05, classes, hidden, seed=5)
    agg = torch.zeros(ctx.nw, dtype=torch.float32, device="cuda")
    worst = 0.0
    for j in range(25 if K < 64 else 8):
        if variant not in ("k_async", "k_batch_async"):
            ctx.set_params(tr.params())
        ctx.step(agg)
        worst = max(worst, rel(agg.cpu().numpy(), tr.step()))
    print(f"worst per-step MLP gradient error {worst:.3e}")
    assert worst <= MLP_GRAD_TOL, worst
    assert_trace_equal(ctx.trace(), tr.trace())
    ctx.close()


def test_mlp_kasync_training_run(ssgd, oracle, torch_cuda):
    """Scaled copy of config 4 (d=512, hidden 128, 10 classes, P=32, m=64, K=4): 150 updates free-running."""
    X, y = synth.mixture_data(4000, 512, 10, seed=6)
    ctx, tr = _mlp_pair(ssgd, oracle, torch_cuda, X, y, 32, 4, 64, "k_async", ("shifted_exp", 0.5, 1.0), 0.05, 10, 128, seed=1)
    ctx.run(150)
    tr.run(150)
    assert_trace_equal(ctx.trace(), tr.trace())
    pr = rel(ctx.params(), tr.params())
    print(f"MLP parameter error after 150 updates {pr:.3e}")
    assert pr <= MLP_PARAM_TOL, pr
    assert np.allclose(ctx.trace()["loss"], tr.trace()["loss"], rtol=5e-3, atol=1e-4)
    ctx.close()


@pytest.mark.parametrize("variant,P,K", [("k_sync", 8, 3), ("k_batch_sync", 8, 5), ("k_batch_async", 8, 3), ("k_async", 8, 6)])
def test_mlp_long_call_takes_the_schedule_in_pieces(ssgd, oracle, torch_cuda, variant, P, K):
    """One call of 70 updates on a single replica of the network: the schedule is written 16 updates at a time on a
    second stream and the gradient kernels take every piece's trace rows from host copies as they arrive -- for every
    variant, also the ones whose updates are launched one after the other (K-async with K = 6 of 8 workers consumes
    gradients of the updating version in most updates, so it is one of them)."""
    X, y = synth.mixture_data(1500, 256, 10, seed=12)
    ctx, tr = _mlp_pair(ssgd, oracle, torch_cuda, X, y, P, K, 32, variant, ("shifted_exp", 0.5, 1.0), 0.05, 10, 128, seed=9)
    ctx.run(70)
    tr.run(70)
    assert_trace_equal(ctx.trace(), tr.trace())
    pr = rel(ctx.params(), tr.params())
    assert pr <= MLP_PARAM_TOL, pr
    assert np.allclose(ctx.trace()["loss"], tr.trace()["loss"], rtol=5e-3, atol=1e-4)
    ctx.close()


def test_mlp_replicas_are_independent_runs(ssgd, oracle, torch_cuda):
    """Three replicas of the network in one context (they run beside each other on streams of their own): each follows
    the oracle's run with its replica index, through a change of K by plateau doubling, and a snapshot taken half-way
    resumes all of them."""
    torch = torch_cuda
    X, y = synth.mixture_data(3000, 256, 10, seed=8)
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.5, 1.0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ada = dict(mode=1, K0=2, Kmax=8, window=20, rel_tol=0.3)
    ctx = ssgd.Context("mlp2", Xd, yd, 12, 2, 32, "k_async", gd, 0.05, seed=7, classes=10, hidden=128, bf16=1, adasync=ada,
                       replicas=3)
    ctx.run(60)
    snap = ctx.get_state()
    ctx.run(60)
    finals = []
    M = oracle.Model("mlp2", X, y, classes=10, hidden=128, bf16=1)
    for r in range(3):
        tr = oracle.Trainer(M, 12, 2, 32, "k_async", od, 0.05, seed=7, adasync=ada, replica=r)
        tr.run(120)
        assert_trace_equal(ctx.trace(r), tr.trace())
        pr = rel(ctx.params(r), tr.params())
        assert pr <= MLP_PARAM_TOL, (r, pr)
        fo = M.full_loss(ctx.params(r))
        assert abs(ctx.full_loss(r) - fo) <= 2e-3 * max(1.0, abs(fo))
        finals.append(ctx.params(r).copy())
    assert not np.array_equal(finals[0], finals[1])
    ctx.set_state(snap)
    ctx.run(60)
    for r in range(3):
        assert np.array_equal(ctx.params(r), finals[r])
    ctx.close()


@pytest.mark.parametrize("P,K", [(8, 2), (128, 32)])
def test_mlp_overlapped_updates_match_updates_one_after_the_other(ssgd, torch_cuda, P, K):
    """A single K-async replica overlaps the forward half of an update with the backward halves of its neighbours in
    every piece of a run where at most a quarter of the updates consume a gradient of their own version; the first
    replica of a two-replica context takes the same run with one update's launches after the other's.  Same trace,
    same losses, bit-identical parameters.  With 8 workers and K = 2 most consumed gradients were started one to four
    versions back, some at the very version that consumes them, so every kind of wait between the halves occurs; with
    128 workers and K = 32 the backward half is the split contraction with its two update kernels."""
    torch = torch_cuda
    X, y = synth.mixture_data(2000, 256, 10, seed=4)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    gd = ssgd.delay_dist("shifted_exp", 0.5, 1.0)
    runs = []
    for replicas in (1, 2):
        ctx = ssgd.Context("mlp2", Xd, yd, P, K, 32, "k_async", gd, 0.05, seed=11, classes=10, hidden=128, bf16=1,
                           replicas=replicas)
        ctx.run(7); ctx.run(150); ctx.run(43)
        runs.append((ctx.trace(0), ctx.params(0).copy()))
        ctx.close()
    (t1, p1), (t2, p2) = runs
    staleness = t1["staleness"][:, :K]
    # the pieces the three calls are run in (64 updates at most) and the library's rule for overlapping one
    overlapped = []
    for a, b in ((0, 7), (7, 71), (71, 135), (135, 157), (157, 200)):
        own = int((staleness[a:b] == 0).any(axis=1).sum())
        if 4 * own <= b - a:
            overlapped.append(staleness[a:b])
    assert len(overlapped) >= 3
    seen = np.concatenate(overlapped)
    if P == 8:
        assert (seen == 0).any() and (seen == 1).any() and (seen >= 3).any()
    for key in ("t", "K", "sel", "staleness", "loss"):
        assert np.array_equal(t1[key], t2[key]), key
    assert np.array_equal(p1, p2)


def test_mlp_kbatch_async_training_run_with_plateau_doubling(ssgd, oracle, torch_cuda):
    """K-batch-async on the MLP, free-running for 120 updates while AdaSync doubles K (2 -> 8) on plateaus: the slot
    of every mini-batch in flight survives the changes of K."""
    X, y = synth.mixture_data(3000, 256, 10, seed=8)
    ada = {"mode": 1, "K0": 2, "Kmax": 8, "window": 15, "rel_tol": 0.5}
    ctx, tr = _mlp_pair(ssgd, oracle, torch_cuda, X, y, 12, 2, 32, "k_batch_async", ("shifted_exp", 0.5, 1.0), 0.05, 10, 128,
                        seed=3, adasync=ada)
    ctx.run(50); ctx.run(70)
    tr.run(120)
    assert_trace_equal(ctx.trace(), tr.trace())
    assert ctx.trace()["K"].max() > 2
    pr = rel(ctx.params(), tr.params())
    print(f"MLP K-batch-async parameter error after 120 updates {pr:.3e}")
    assert pr <= MLP_PARAM_TOL, pr
    assert np.allclose(ctx.trace()["loss"], tr.trace()["loss"], rtol=5e-3, atol=1e-4)
    ctx.close()


def test_mlp_adasync_plateau_doubling(ssgd, oracle, torch_cuda):
    """AdaSync on the MLP (config 4's controller, scaled: windows of 20 updates, K 2 -> 16, P=16): K changes
    at the same updates as in the oracle, and the schedule stays bit-exact through the changes."""
    X, y = synth.mixture_data(3000, 256, 10, seed=8)
    ada = dict(mode=1, K0=2, Kmax=16, window=20, rel_tol=0.01)
    ctx, tr = _mlp_pair(ssgd, oracle, torch_cuda, X, y, 16, 2, 32, "k_async", ("shifted_exp", 0.5, 1.0), 0.05, 10, 128,
                        seed=2, adasync=ada)
    ctx.run(160)
    tr.run(160)
    g, o = ctx.trace(), tr.trace()
    assert np.array_equal(g["K"], o["K"]), (g["K"], o["K"])
    assert len(set(g["K"].tolist())) >= 2      # K did change
    assert_trace_equal(g, o)
    assert rel(ctx.params(), tr.params()) <= 5e-3
    ctx.close()


def test_config4_mlp_full_size_first_updates(ssgd, oracle, torch_cuda, mixture_full):
    """Config 4 at its real shape (d=3072, 512 hidden units, 10 classes, N=50000, P=256, m=64, K=8, shifted-Exp):
    update 0 starts all 256 workers (16384 rows through the large-tile contraction); three per-step aggregates
    and then ten free-running updates against the oracle (a longer horizon costs the oracle a second per update)."""
    torch = torch_cuda
    X, y, Xd, yd = mixture_full
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.5, 1.0))
    ada = dict(mode=1, K0=8, Kmax=256, window=200, rel_tol=0.01)
    ctx = ssgd.Context("mlp2", Xd, yd, 256, 8, 64, "k_async", gd, 0.05, seed=0, classes=10, hidden=512, bf16=1, adasync=ada)
    tr = oracle.Trainer(oracle.Model("mlp2", X, y, classes=10, hidden=512, bf16=1), 256, 8, 64, "k_async", od, 0.05,
                        seed=0, adasync=ada)
    assert np.array_equal(ctx.params(), tr.params())
    agg = torch.zeros(ctx.nw, dtype=torch.float32, device="cuda")
    worst = 0.0
    for j in range(3):
        ctx.step(agg)
        worst = max(worst, rel(agg.cpu().numpy(), tr.step()))
    ctx.run(10)
    tr.run(10)
    assert_trace_equal(ctx.trace(), tr.trace())
    pr = rel(ctx.params(), tr.params())
    print(f"config 4 full size: worst per-step gradient error {worst:.3e}, parameter error after 13 updates {pr:.3e}")
    assert worst <= MLP_GRAD_TOL, worst
    assert pr <= MLP_PARAM_TOL, pr
    assert np.allclose(ctx.trace()["loss"], tr.trace()["loss"], rtol=5e-3, atol=1e-4)
    ctx.close()


def test_config4_mlp_full_size_large_K(ssgd, oracle, torch_cuda, mixture_full):
    """Config 4 at its real shape with K forced to the values AdaSync's doubling ends at (Algorithm 1 raises K up
    to P): two updates at K=64 and one at K=256, each averaged gradient against the oracle's.  From K=64 on the
    first-layer gradient runs as the split contraction (128 x 128 tiles over 512 x 3072 outputs, shares of the
    consumed slots added in order) followed by the separate update kernel."""
    torch = torch_cuda
    X, y, Xd, yd = mixture_full
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.5, 1.0))
    ada = dict(mode=1, K0=8, Kmax=256, window=200, rel_tol=0.01)
    ctx = ssgd.Context("mlp2", Xd, yd, 256, 8, 64, "k_async", gd, 0.05, seed=0, classes=10, hidden=512, bf16=1, adasync=ada)
    tr = oracle.Trainer(oracle.Model("mlp2", X, y, classes=10, hidden=512, bf16=1), 256, 8, 64, "k_async", od, 0.05,
                        seed=0, adasync=ada)
    agg = torch.zeros(ctx.nw, dtype=torch.float32, device="cuda")
    errs = []
    for K in (64, 64, 256):
        ctx.force_K(K)
        tr.force_K(K)
        ctx.step(agg)
        errs.append(rel(agg.cpu().numpy(), tr.step()))
    assert_trace_equal(ctx.trace(), tr.trace())
    assert list(ctx.trace()["K"]) == [64, 64, 256]
    pr = rel(ctx.params(), tr.params())
    print(f"config 4 full size, K = 64, 64, 256: per-step gradient errors {errs}, parameter error {pr:.3e}")
    assert max(errs) <= MLP_GRAD_TOL, errs
    assert pr <= MLP_PARAM_TOL, pr
    ctx.close()


def test_exchange_fallback_without_shared_l2(ssgd, oracle, torch_cuda, monkeypatch):
    """The cluster exchange has two protocols: through the L2 of one XCD (data words polled directly) and, for a
    cluster that is spread over XCDs, released stores with an arrival counter.  The second one is forced here."""
    monkeypatch.setenv("SSGD_EXCHANGE", "fenced")
    X, y = synth.mixture_data(1500, 640, 10, seed=1)
    _run_pair(ssgd, oracle, torch_cuda, "softmax", X, y, 8, 2, 32, "k_async", ("shifted_exp", 0.5, 1.0), 0.05, 150, seed=4,
              classes=10)


@pytest.mark.parametrize("kind,variant,P,K,m,d,classes", [
    ("lsq", "k_async", 6, 3, 16, 300, 1),          # least squares on the single-tile kernel, ragged second slice
    ("lsq", "k_sync", 5, 4, 10, 516, 1),           # m not a multiple of 4 (padded rows), three slices
    ("softmax", "k_async", 7, 4, 10, 260, 15),     # 15 classes (the most the single-tile kernel takes), 48 of 64 rows used
    ("softmax", "k_batch_sync", 4, 6, 8, 1028, 7), # a worker contributes twice; five slices
])
def test_single_tile_kernel_shapes(ssgd, oracle, torch_cuda, kind, variant, P, K, m, d, classes):
    if kind == "lsq":
        X, y, _ = synth.lsq_data(1200, d, 5)
    else:
        X, y = synth.mixture_data(1200, d, classes, seed=5)
    _run_pair(ssgd, oracle, torch_cuda, kind, X, y, P, K, m, variant, ("shifted_exp", 0.5, 1.0), 0.02, 100, seed=6,
              classes=classes)


def test_more_replicas_than_one_launch_holds(ssgd, oracle, torch_cuda):
    """45 replicas of a 12-slice cluster need several launches (16 + 16 + 13); zero updates are a no-op."""
    torch = torch_cuda
    X, y = synth.mixture_data(3000, 3072, 10, seed=7)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.5, 1.0))
    ctx = ssgd.Context("softmax", Xd, yd, 8, 2, 32, "k_async", gd, 0.05, seed=2, classes=10, replicas=45)
    ctx.run(0)
    assert ctx.updates == 0
    ctx.run(60)
    for r in (0, 39, 40, 44):
        tr = oracle.Trainer(oracle.Model("softmax", X, y, classes=10), 8, 2, 32, "k_async", od, 0.05, seed=2, replica=r)
        tr.run(60)
        assert_trace_equal(ctx.trace(r), tr.trace())
        assert rel(ctx.params(r), tr.params()) <= FP32_PARAM_TOL
    ctx.close()


def test_k_async_kernel_hands_spread_clusters_to_the_fenced_exchange(ssgd, oracle, torch_cuda, monkeypatch):
    """The K-async steady-state kernel exchanges through the L2 of one XCD.  A cluster that finds its workgroups on
    several XCDs leaves its replica untouched and flags it, and the host runs those replicas through the kernel that
    can exchange across XCDs.  Here the odd replicas are told that they are spread out (a host-side switch; every
    kernel exits normally): all replicas must still follow the oracle."""
    torch = torch_cuda
    monkeypatch.setenv("SSGD_DEBUG_FLAGS", "2")
    X, y = synth.mixture_data(2000, 1280, 10, seed=11)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.5, 1.0))
    ctx = ssgd.Context("softmax", Xd, yd, 8, 2, 32, "k_async", gd, 0.05, seed=5, classes=10, replicas=5)
    ctx.run(50)
    ctx.run(40)
    for r in (0, 1, 3, 4):
        tr = oracle.Trainer(oracle.Model("softmax", X, y, classes=10), 8, 2, 32, "k_async", od, 0.05, seed=5, replica=r)
        tr.run(90)
        assert_trace_equal(ctx.trace(r), tr.trace())
        assert rel(ctx.params(r), tr.params()) <= FP32_PARAM_TOL
    ctx.close()


def test_parked_gradients_with_two_workgroups_per_cu(ssgd, oracle, torch_cuda, monkeypatch):
    """K-async through the kernel that parks gradients in HBM, 40 replicas of twelve slices in one launch (two
    workgroups per CU): replicas from both halves of the launch follow the oracle through updates that consume parked
    gradients.  (A 16-byte store that lost its data in the second workgroup of a CU once showed up exactly here.)"""
    torch = torch_cuda
    monkeypatch.setenv("SSGD_KERNEL", "tile")
    X, y = synth.mixture_data(3000, 3072, 10, seed=7)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.5, 1.0))
    ctx = ssgd.Context("softmax", Xd, yd, 8, 2, 32, "k_async", gd, 0.05, seed=2, classes=10, replicas=40)
    ctx.run(40)
    for r in (0, 8, 20, 37, 39):
        tr = oracle.Trainer(oracle.Model("softmax", X, y, classes=10), 8, 2, 32, "k_async", od, 0.05, seed=2, replica=r)
        tr.run(40)
        assert_trace_equal(ctx.trace(r), tr.trace())
        assert rel(ctx.params(r), tr.params()) <= FP32_PARAM_TOL
    ctx.close()


@pytest.mark.parametrize("kind,variant,P,K,m,d,classes", [
    ("lsq", "k_batch_sync", 3, 5, 70, 132, 1),     # records of 72 rows straddle the 64-row tiles; 5.6 tiles
    ("softmax", "k_sync", 6, 5, 30, 516, 10),      # 2.5 tiles of padded 32-row records, three slices
    ("softmax", "k_batch_sync", 5, 12, 64, 260, 3),  # twelve full tiles, a worker contributes several times
])
def test_iterations_of_several_tiles(ssgd, oracle, torch_cuda, kind, variant, P, K, m, d, classes):
    """Synchronous iterations whose K mini-batches do not fit one 64-row tile run tile by tile in the steady-state
    kernel, the update after the last tile."""
    if kind == "lsq":
        X, y, _ = synth.lsq_data(1200, d, 8)
    else:
        X, y = synth.mixture_data(1200, d, classes, seed=8)
    _run_pair(ssgd, oracle, torch_cuda, kind, X, y, P, K, m, variant, ("pareto", 2.5, 1.0), 0.02, 60, seed=9,
              classes=classes, check_steps=20)


def test_adasync_ksync_rule_with_growing_tile_count(ssgd, oracle, torch_cuda):
    """K-sync under the paper's rule for K (Appendix D): K grows from 2 to 16 during the run, so the iterations go
    from one tile to two; trace and parameters against the oracle."""
    torch = torch_cuda
    X, y, _ = synth.lsq_data(512, 16, 3)
    gd, od = dist_pair(ssgd, oracle, ("exp", 1.0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ada = dict(mode=3, K0=2, Kmax=16, interval_t=6.0)
    ctx = ssgd.Context("lsq", Xd, yd, 16, 2, 8, "k_sync", gd, 0.03, seed=2, adasync=ada)
    tr = oracle.Trainer(oracle.Model("lsq", X, y), 16, 2, 8, "k_sync", od, 0.03, seed=2, adasync=ada)
    ctx.run(300)
    tr.run(300)
    g, o = ctx.trace(), tr.trace()
    assert o["K"][-1] > 8
    assert_trace_equal(g, o)
    assert np.allclose(g["loss"], o["loss"], rtol=FP32_LOSS_RTOL, atol=1e-6)
    assert rel(ctx.params(), tr.params()) <= FP32_PARAM_TOL
    ctx.close()


# ------------------------------------------------------------------------------- worker state, snapshot and resume

def test_workers_in_flight_bit_exact(ssgd, oracle, torch_cuda):
    """tau_i and f_i of every K-async worker after a run, against the oracle's event state."""
    torch = torch_cuda
    X, y, _ = synth.lsq_data(256, 8, 1)
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.2, 1.0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ctx = ssgd.Context("lsq", Xd, yd, 24, 5, 4, "k_async", gd, 0.01, seed=11)
    tr = oracle.Trainer(oracle.Model("lsq", X, y), 24, 5, 4, "k_async", od, 0.01, seed=11)
    ctx.run(333)
    tr.run(333)
    g = ctx.workers()
    otau, ofinish = tr.workers()
    assert np.array_equal(g["tau"].astype(np.int64), otau)
    assert np.array_equal(g["finish"], ofinish)
    ctx.close()
    sync = ssgd.Context("lsq", Xd, yd, 4, 2, 4, "k_sync", gd, 0.01, seed=11)
    with pytest.raises(ssgd.SsgdError):
        sync.workers()
    sync.close()


@pytest.mark.parametrize("kind,variant,P,K,m,d,classes,ada", [
    ("softmax", "k_async", 8, 2, 32, 512, 10, None),                 # steady-state kernel, parked gradients in flight
    ("softmax", "k_batch_sync", 5, 6, 40, 260, 4, None),             # iterations of several tiles
    ("lsq", "k_async", 12, 2, 6, 30, 1, dict(mode=1, K0=2, Kmax=12, window=16, rel_tol=0.5)),   # general kernel, AdaSync window open
])
def test_snapshot_resume_continues_the_same_run(ssgd, oracle, torch_cuda, kind, variant, P, K, m, d, classes, ada):
    """A run that is snapshotted and resumed in a new context is the run that was never interrupted: identical trace
    and parameters, bit for bit (every sum on the device is taken in a fixed order); the oracle agrees with both."""
    torch = torch_cuda
    if kind == "lsq":
        X, y, _ = synth.lsq_data(900, d, 12)
    else:
        X, y = synth.mixture_data(900, d, classes, seed=12)
    gd, od = dist_pair(ssgd, oracle, ("exp", 1.0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    mk = lambda: ssgd.Context(kind, Xd, yd, P, K, m, variant, gd, 0.03, seed=13, classes=classes, replicas=3, adasync=ada)
    a = mk()
    a.run(57)
    blob = a.get_state()
    a.run(43)
    b = mk()
    b.run(5)                 # whatever the receiving context did before is replaced
    b.set_state(blob)
    assert b.updates == 57
    b.run(43)
    for r in range(3):
        ta, tb = a.trace(r), b.trace(r)
        for key in ta:
            assert np.array_equal(ta[key], tb[key]), (r, key)
        assert np.array_equal(a.params(r), b.params(r)), r
    tr = oracle.Trainer(oracle.Model(kind, X, y, classes=classes), P, K, m, variant, od, 0.03, seed=13, replica=2, adasync=ada)
    tr.run(100)
    assert_trace_equal(b.trace(2), tr.trace())
    assert rel(b.params(2), tr.params()) <= FP32_PARAM_TOL
    # a snapshot of another configuration is refused and leaves the context as it was
    other = ssgd.Context(kind, Xd, yd, P, K, m, variant, gd, 0.03, seed=14, classes=classes, replicas=3, adasync=ada)
    with pytest.raises(ssgd.SsgdError):
        other.set_state(blob)
    assert other.updates == 0
    for c in (a, b, other):
        c.close()


def test_malformed_snapshots_leave_the_context_unchanged(ssgd, oracle, torch_cuda):
    """A truncated buffer, a header that claims more updates than the buffer holds, or one whose size does not
    fit this configuration is refused with SSGD_EINVAL before the context is touched: the run goes on as if
    nothing had been tried."""
    torch = torch_cuda
    X, y = synth.mixture_data(800, 320, 10, seed=3)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.5, 1.0))
    ctx = ssgd.Context("softmax", Xd, yd, 8, 2, 32, "k_async", gd, 0.05, seed=1, classes=10)
    ctx.run(20)
    good = ctx.get_state()
    ctx.run(15)
    hdr_j = 8 + 8 + 12 * 4 + 2 * 8        # offset of the update count in the header: magic, size, 12 ints, N, nw
    assert int(np.frombuffer(good, dtype=np.int64, count=1, offset=hdr_j)[0]) == 20
    def with_j(v):
        b = good.copy()
        b[hdr_j:hdr_j + 8] = np.frombuffer(np.int64(v).tobytes(), dtype=np.uint8)
        return b
    bad = [good[:-64].copy(),                                     # truncated
           with_j(2 ** 40), with_j(-3), with_j(19),               # update counts the buffer cannot hold / does not match
           np.frombuffer(b"SSGDST01" + bytes(40), dtype=np.uint8)]   # shorter than a header
    for b in bad:
        with pytest.raises(ssgd.SsgdError) as ei:
            ctx.set_state(b)
        assert ei.value.status == ssgd.EINVAL
        assert ctx.updates == 35
    ctx.run(10)
    tr = oracle.Trainer(oracle.Model("softmax", X, y, classes=10), 8, 2, 32, "k_async", od, 0.05, seed=1)
    tr.run(45)
    assert_trace_equal(ctx.trace(), tr.trace())
    assert rel(ctx.params(), tr.params()) <= FP32_PARAM_TOL
    ctx.set_state(good)                                           # and a good snapshot is still accepted
    assert ctx.updates == 20
    ctx.close()


@pytest.mark.parametrize("variant,K", [("k_async", 2), ("k_batch_async", 4)])
def test_mlp_snapshot_resume(ssgd, oracle, torch_cuda, variant, K):
    torch = torch_cuda
    X, y = synth.mixture_data(600, 256, 5, seed=15)
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.5, 1.0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    mk = lambda: ssgd.Context("mlp2", Xd, yd, 6, K, 16, variant, gd, 0.05, seed=16, classes=5, hidden=128, bf16=1)
    a = mk()
    a.run(9)
    blob = a.get_state()
    a.run(7)
    b = mk()
    b.set_state(blob)
    b.run(7)
    ta, tb = a.trace(), b.trace()
    for key in ta:
        assert np.array_equal(ta[key], tb[key]), key
    assert np.array_equal(a.params(), b.params())
    a.close(); b.close()


def test_mlp_snapshot_resume_through_overlapped_updates(ssgd, torch_cuda):
    """Snapshot and resume where a single K-async replica overlaps its updates (calls of 40 updates, 8 workers, K = 2):
    the operand copies of the parameters that the overlapped launches keep per version are rebuilt from the
    snapshot's parameters, and the resumed run is the original one bit by bit."""
    torch = torch_cuda
    X, y = synth.mixture_data(1500, 256, 10, seed=21)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    gd = ssgd.delay_dist("shifted_exp", 0.5, 1.0)
    mk = lambda: ssgd.Context("mlp2", Xd, yd, 8, 2, 32, "k_async", gd, 0.05, seed=23, classes=10, hidden=128, bf16=1)
    a = mk()
    a.run(40)
    blob = a.get_state()
    a.run(40)
    b = mk()
    b.run(5)                 # a different past, replaced by the snapshot
    b.set_state(blob)
    b.run(40)
    ta, tb = a.trace(), b.trace()
    for key in ta:
        assert np.array_equal(ta[key], tb[key]), key
    assert np.array_equal(a.params(), b.params())
    a.close(); b.close()


# ------------------------------------------------------------------------------- K-batch-async

@pytest.mark.parametrize("kind,P,K,m,d,classes,spec", [
    ("softmax", 8, 2, 32, 320, 10, ("shifted_exp", 0.5, 1.0)),   # the shape of config 1, two slices
    ("lsq", 6, 4, 10, 132, 1, ("exp", 1.0)),                      # padded mini-batches, five records per tile
    ("softmax", 5, 7, 16, 260, 3, ("pareto", 2.5, 1.0)),          # K > P: workers push several times per update
    ("softmax", 12, 3, 64, 516, 15, ("exp", 2.5)),                # one record per tile: 14 tiles at version 0
    ("lsq", 4, 2, 16, 64, 1, ("exp", 1.0)),                       # config 0's shape: a single, mostly empty slice
    ("softmax", 6, 3, 8, 20, 4, ("shifted_exp", 0.5, 1.0)),       # d = 20
    ("softmax", 64, 16, 32, 320, 10, ("pareto", 2.5, 1.0)),       # config 2's workers and K: 79 records at version 0
    ("lsq", 200, 3, 8, 64, 1, ("exp", 1.0)),                      # 202 records at version 0, 8 per tile
    ("softmax", 130, 32, 64, 260, 3, ("exp", 1.0)),               # one record per tile, 161 tiles at version 0, K = 32
    ("softmax", 6, 4, 128, 260, 10, ("shifted_exp", 0.5, 1.0)),   # mini-batches of two tiles
    ("lsq", 5, 3, 72, 132, 1, ("exp", 1.0)),                      # 72 rows: a full tile and one of 8 rows per record
    ("softmax", 4, 6, 200, 516, 7, ("pareto", 2.5, 1.0)),         # four tiles per record (the last of 8 rows), K > P
    ("softmax", 64, 16, 128, 320, 10, ("pareto", 2.5, 1.0)),      # config 2's P, K and m: 158 tiles at version 0
    ("softmax", 20, 48, 16, 260, 5, ("exp", 1.0)),                # K = 48 > P: lists longer than 32 entries
    ("lsq", 70, 64, 8, 132, 1, ("shifted_exp", 0.5, 1.0)),        # K = 64, the most a wave's lanes hold
])
def test_kbatch_async_parity(ssgd, oracle, torch_cuda, kind, P, K, m, d, classes, spec):
    """K-batch-async (Sec. 2.2): delays, selections, ordinals and staleness bit for bit, per-update averaged gradients
    and final parameters within tolerance, free-running against the oracle."""
    if kind == "lsq":
        X, y, _ = synth.lsq_data(1000, d, 21)
    else:
        X, y = synth.mixture_data(1000, d, classes, seed=21)
    _run_pair(ssgd, oracle, torch_cuda, kind, X, y, P, K, m, "k_batch_async", spec, 0.03, 150, seed=22, classes=classes,
              check_steps=50)


def test_kbatch_async_long_schedule_and_workers(ssgd, oracle, torch_cuda):
    """2000 updates with P = 40 workers and K = 9: the trace and the workers' in-flight state (tau_i, f_i) against
    the oracle, then a snapshot taken mid-run resumes to the same end."""
    torch = torch_cuda
    X, y, _ = synth.lsq_data(400, 132, 23)
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.2, 1.0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    mk = lambda: ssgd.Context("lsq", Xd, yd, 40, 9, 2, "k_batch_async", gd, 0.01, seed=24)
    ctx = mk()
    tr = oracle.Trainer(oracle.Model("lsq", X, y), 40, 9, 2, "k_batch_async", od, 0.01, seed=24)
    ctx.run(1200)
    blob = ctx.get_state()
    ctx.run(800)
    tr.run(2000)
    assert_trace_equal(ctx.trace(), tr.trace())
    g = ctx.workers()
    otau, ofinish = tr.workers()
    assert np.array_equal(g["tau"].astype(np.int64), otau)
    assert np.array_equal(g["finish"], ofinish)
    assert rel(ctx.params(), tr.params()) <= FP32_PARAM_TOL
    other = mk()
    other.set_state(blob)
    other.run(800)
    assert np.array_equal(other.params(), ctx.params())
    ctx.close(); other.close()


def test_kbatch_async_unsupported_shapes_are_refused(ssgd, torch_cuda):
    torch = torch_cuda
    X, y, _ = synth.lsq_data(64, 66, 1)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    for P, K, m, cols in ((4, 2, 8, 66), (8, 65, 8, 64)):
        # d % 4 != 0; K > 64
        Xc = Xd[:, :cols].contiguous()
        with pytest.raises(ssgd.SsgdError):
            ssgd.Context("lsq", Xc, yd, P, K, m, "k_batch_async", ssgd.delay_dist("exp", 1.0), 0.01)


# ------------------------------------------------------------------------------- objective over the whole data set

@pytest.mark.parametrize("kind,N,d,classes", [
    ("softmax", 1500, 320, 10), ("softmax", 1001, 132, 3), ("softmax", 37, 64, 16), ("lsq", 4096, 64, 1),
    ("lsq", 777, 100, 1), ("softmax", 2000, 3072, 10),
])
def test_full_objective_against_the_oracle(ssgd, oracle, torch_cuda, kind, N, d, classes):
    """F(w) of Eq. (1) after some training, and at w = 0 where the softmax objective is ln(classes) for any data."""
    torch = torch_cuda
    if kind == "lsq":
        X, y, _ = synth.lsq_data(N, d, 41)
    else:
        X, y = synth.mixture_data(N, d, classes, seed=41)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ctx = ssgd.Context(kind, Xd, yd, 4, 2, 8, "k_sync", ssgd.delay_dist("exp", 1.0), 0.05 if kind == "softmax" else 0.01,
                       seed=42, classes=classes, replicas=2)
    M = oracle.Model(kind, X, y, classes=classes)
    f0 = ctx.full_loss(0)
    assert abs(f0 - M.full_loss(np.zeros(ctx.nw, dtype=np.float32))) <= 1e-6 * max(1.0, abs(f0))
    if kind == "softmax":
        assert abs(f0 - math.log(classes)) < 1e-6
    ctx.run(30)
    for r in (0, 1):
        g, o = ctx.full_loss(r), M.full_loss(ctx.params(r))
        assert abs(g - o) <= 2e-6 * max(1.0, abs(o)), (r, g, o)
    assert ctx.full_loss(0) != ctx.full_loss(1)
    ctx.close()


@pytest.mark.parametrize("N,d,classes,hidden,variant", [
    (1000, 256, 10, 128, "k_async"),       # 16 slots, the last one ragged
    (20000, 128, 5, 256, "k_sync"),        # 313 slots: two passes of the evaluation buffers, the large forward tiles
    (37, 128, 16, 128, "k_async"),         # less than one slot
])
def test_full_objective_of_the_two_layer_network(ssgd, oracle, torch_cuda, N, d, classes, hidden, variant):
    """F(w) of Eq. (1) for the MLP with the forward pass of the trainer (bf16 operands), against the oracle's
    objective with the same rounding; evaluating in the middle of a K-async run must not disturb the run."""
    X, y = synth.mixture_data(N, d, classes, seed=43)
    ctx, tr = _mlp_pair(ssgd, oracle, torch_cuda, X, y, 8, 2, 16, variant, ("exp", 1.0), 0.05, classes, hidden, seed=5)
    M = oracle.Model("mlp2", X, y, classes=classes, hidden=hidden, bf16=1)
    g, o = ctx.full_loss(0), M.full_loss(ctx.params())
    assert abs(g - o) <= 1e-5 * max(1.0, abs(o)), (g, o)
    ctx.run(20)
    g, o = ctx.full_loss(0), M.full_loss(ctx.params())
    assert abs(g - o) <= 1e-5 * max(1.0, abs(o)), (g, o)
    assert ctx.full_loss(0) == g                      # repeatable
    ctx.run(20)                                       # the mini-batches in flight were left alone
    tr.run(40)
    assert_trace_equal(ctx.trace(), tr.trace())
    assert rel(ctx.params(), tr.params()) <= MLP_PARAM_TOL
    other, _ = _mlp_pair(ssgd, oracle, torch_cuda, X, y, 8, 2, 16, variant, ("exp", 1.0), 0.05, classes, hidden, seed=5)
    other.run(40)
    assert np.array_equal(other.params(), ctx.params())
    ctx.close(); other.close()


@pytest.mark.parametrize("kind,N,d,classes", [
    ("softmax", 1500, 320, 10), ("softmax", 1001, 132, 3), ("softmax", 37, 64, 16), ("lsq", 4096, 64, 1),
    ("lsq", 777, 100, 1), ("softmax", 20000, 3072, 10),
])
def test_full_gradient_against_the_oracle(ssgd, oracle, torch_cuda, kind, N, d, classes):
    """grad F of Eq. (1) at w = 0 and after some training, both replicas, against the oracle's fp64 gradient."""
    torch = torch_cuda
    if kind == "lsq":
        X, y, _ = synth.lsq_data(N, d, 44)
    else:
        X, y = synth.mixture_data(N, d, classes, seed=44)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ctx = ssgd.Context(kind, Xd, yd, 4, 2, 8, "k_sync", ssgd.delay_dist("exp", 1.0), 0.05 if kind == "softmax" else 0.01,
                       seed=45, classes=classes, replicas=2)
    M = oracle.Model(kind, X, y, classes=classes)
    assert rel(ctx.full_gradient(0), M.full_grad(np.zeros(ctx.nw, dtype=np.float32))) <= 1e-5
    ctx.run(25)
    for r in (0, 1):
        e = rel(ctx.full_gradient(r), M.full_grad(ctx.params(r)))
        assert e <= 1e-5, (r, e)
    assert not np.array_equal(ctx.full_gradient(0), ctx.full_gradient(1))
    ctx.close()


def test_staleness_gamma_estimate_for_the_network(ssgd, torch_cuda):
    """The same estimate on the two-layer network with two replicas: zero for K-sync, positive for K-async."""
    from paper_2003_10579_amd import staleness_gamma
    torch = torch_cuda
    X, y = synth.mixture_data(1500, 256, 5, seed=9)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    kw = dict(kind="mlp2", classes=5, hidden=128, bf16=1)
    sync = staleness_gamma.gamma_estimate(ssgd, Xd, yd, 8, 4, 16, "k_sync", ("exp", 1.0), 0.05, 12, 2, seed=3, **kw)
    assert sync["gamma"] == 0.0 and sync["p0"] == 1.0
    asy = staleness_gamma.gamma_estimate(ssgd, Xd, yd, 8, 2, 16, "k_async", ("exp", 1.0), 0.05, 25, 2, seed=3, **kw)
    assert asy["gamma"] > 0.0 and 0.0 < asy["p0"] < 1.0


@pytest.mark.parametrize("N,d,hidden,classes", [(1000, 256, 128, 10), (20000, 384, 256, 7)])
def test_full_gradient_of_the_network_against_the_oracle(ssgd, oracle, torch_cuda, N, d, hidden, classes):
    """grad F of Eq. (1) for the two-layer network, at the initial parameters and after some training (a ragged last
    block of rows; the second shape takes more than one block of 256 slots), against the oracle's gradient; the
    parameters, the trace and the mini-batches in flight are untouched by the call."""
    torch = torch_cuda
    X, y = synth.mixture_data(N, d, classes, seed=46)
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.5, 1.0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ctx = ssgd.Context("mlp2", Xd, yd, 8, 2, 32, "k_async", gd, 0.05, seed=47, classes=classes, hidden=hidden, bf16=1)
    M = oracle.Model("mlp2", X, y, classes=classes, hidden=hidden, bf16=1)
    tr = oracle.Trainer(M, 8, 2, 32, "k_async", od, 0.05, seed=47)
    e0 = rel(ctx.full_gradient(0), M.full_grad(ctx.params(0)))
    ctx.run(20); tr.run(20)
    w = ctx.params(0).copy()
    e1 = rel(ctx.full_gradient(0), M.full_grad(w))
    print(f"network full gradient: {e0:.3e} at w_0, {e1:.3e} after 20 updates")
    assert e0 <= MLP_GRAD_TOL and e1 <= MLP_GRAD_TOL, (e0, e1)
    assert np.array_equal(ctx.params(0), w)
    ctx.run(20); tr.run(20)                       # the run goes on as if the call had not happened
    assert_trace_equal(ctx.trace(), tr.trace())
    assert rel(ctx.params(0), tr.params()) <= MLP_PARAM_TOL
    ctx.close()


def test_staleness_gamma_estimate(ssgd, oracle, torch_cuda):
    """gamma of the staleness bound (fifth assumption of Sec. 4.1) from the driver: zero for a synchronous variant (every gradient is fresh), positive and
    growing with the staleness for K-async (K = 1 against K = P / 2 at P = 8), and equal to the same ratio formed
    from the oracle's fp64 gradients at the iterates of the run."""
    from paper_2003_10579_amd import staleness_gamma
    torch = torch_cuda
    X, y, _ = synth.lsq_data(1024, 132, 6)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    spec = ("exp", 1.0)
    sync = staleness_gamma.gamma_estimate(ssgd, Xd, yd, 8, 4, 8, "k_sync", spec, 0.01, 40, 2, seed=3)
    assert sync["gamma"] == 0.0 and sync["p0"] == 1.0
    a1, params = staleness_gamma.gamma_estimate(ssgd, Xd, yd, 8, 1, 8, "k_async", spec, 0.01, 60, 2, seed=3, keep_params=True)
    a4 = staleness_gamma.gamma_estimate(ssgd, Xd, yd, 8, 4, 8, "k_async", spec, 0.01, 60, 2, seed=3)
    assert a1["gamma"] > a4["gamma"] > 0.0, (a1["gamma"], a4["gamma"])
    assert a1["mean_staleness"] > a4["mean_staleness"] and a1["p0"] < a4["p0"]
    # the same statistic from the oracle's gradients and the oracle's own schedule
    M = oracle.Model("lsq", X, y)
    gd, od = dist_pair(ssgd, oracle, spec)
    num = den = 0.0
    used = 0
    for r in range(2):
        tr = oracle.Trainer(M, 8, 1, 8, "k_async", od, 0.01, seed=3, replica=r)
        tr.run(60)
        st = tr.trace()["staleness"]
        g = [M.full_grad(w) for w in params[r]]
        for j in range(60):
            den += float(g[j] @ g[j])
            s = int(st[j, 0])
            num += float((g[j] - g[j - s]) @ (g[j] - g[j - s]))
            used += 1
    want = (num / used) / (den / 120)
    assert abs(a1["gamma"] - want) <= 1e-4 * want, (a1["gamma"], want)


def test_error_runtime_frontier_against_the_oracle(ssgd, oracle, torch_cuda):
    """The four variants at the same K on the same problem (Sec. 3, Table 1).  Every point of the trade-off against
    the oracle, replica by replica: the simulated time t_J bit for bit and the sub-optimality F(w_J) - F* (Sec. 2.3)
    within 1e-3 relative.  Then the orderings: per update K-batch-async is the fastest and K-sync the slowest; the
    synchronous variants only use fresh gradients, the asynchronous ones do not; every run ends above the optimum."""
    from paper_2003_10579_amd import frontier
    torch = torch_cuda
    X, y, _ = synth.lsq_data(2048, 132, 3)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    X64, y64 = X.astype(np.float64), y.astype(np.float64)
    w_opt = np.linalg.solve(X64.T @ X64, X64.T @ y64)
    f_star = 0.5 * float(np.mean((X64 @ w_opt - y64) ** 2))
    recs = frontier.frontier(ssgd, Xd, yd, f_star, 8, [2, 4], 8, 0.01, 300, 6, ("shifted_exp", 1.0, 1.0), seed=1)
    by = {(r["variant"], r["K"]): r for r in recs}
    M = oracle.Model("lsq", X, y)
    od = oracle.Dist("shifted_exp", 1.0, 1.0)
    worst_gap = 0.0
    for (variant, K), rec in by.items():
        for r in range(6):
            tr = oracle.Trainer(M, 8, K, 8, variant, od, 0.01, seed=1, replica=r)
            tr.run(300)
            assert tr.clock == rec["time_by_replica"][r], (variant, K, r)
            gap = M.full_loss(tr.params()) - f_star
            assert gap > 0
            worst_gap = max(worst_gap, abs(rec["gap_by_replica"][r] - gap) / gap)
    print(f"error-runtime trade-off: worst relative difference of F(w_J) - F* from the oracle's {worst_gap:.2e}")
    assert worst_gap <= 1e-3, worst_gap
    for K in (2, 4):
        ts = [by[(v, K)]["time_per_update"] for v in ("k_batch_async", "k_async", "k_sync")]
        assert ts[0] < ts[1] < ts[2], ts
        assert by[("k_batch_sync", K)]["time_per_update"] <= by[("k_sync", K)]["time_per_update"]      # Lemma 2
        for v in ("k_sync", "k_batch_sync"):
            assert by[(v, K)]["p0"] == 1.0 and by[(v, K)]["mean_staleness"] == 0.0
        for v in ("k_async", "k_batch_async"):
            assert 0.0 < by[(v, K)]["p0"] < 1.0 and by[(v, K)]["mean_staleness"] > 0.0
    assert all(r["mean_gap"] > 0 for r in recs)
    # more contributors per update: each update takes longer (Lemma 1, Lemma 3) ...
    assert by[("k_sync", 4)]["time_per_update"] > by[("k_sync", 2)]["time_per_update"]
    # ... and for the asynchronous variants the gradients used are less stale
    assert by[("k_async", 4)]["mean_staleness"] < by[("k_async", 2)]["mean_staleness"]


def test_speedups_of_theorems_1_and_2(ssgd, torch_cuda):
    """Theorem 1 (fully asynchronous against fully synchronous SGD: P (1 + 1/2 + ... + 1/P) for exponential delays) and
    Theorem 2 (K-async against K-batch-async: P E[X_{K:P}] / (K E[X])) from the Monte-Carlo estimator, within 2 %."""
    from paper_2003_10579_amd import speedup
    for rec in speedup.speedups(ssgd, ("exp", 1.0), Ps=(4, 32, 128), trials=100000, seed=3):
        assert abs(rec["sync_over_async"] / rec["theorem1_closed_form"] - 1) < 0.02, rec
        assert abs(rec["k_async_over_k_batch_async"] / rec["theorem2_closed_form"] - 1) < 0.02, rec


def test_kbatch_async_with_plateau_doubling(ssgd, oracle, torch_cuda):
    """AdaSync by plateau doubling on top of K-batch-async: K grows from 1 to 8 during the run (record lists of every
    size, windows closing mid-segment); trace, K sequence and parameters against the oracle."""
    torch = torch_cuda
    X, y = synth.mixture_data(800, 260, 4, seed=51)
    gd, od = dist_pair(ssgd, oracle, ("shifted_exp", 0.2, 1.0))
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    ada = dict(mode=1, K0=1, Kmax=8, window=20, rel_tol=0.5)
    ctx = ssgd.Context("softmax", Xd, yd, 10, 1, 12, "k_batch_async", gd, 0.05, seed=52, classes=4, adasync=ada)
    tr = oracle.Trainer(oracle.Model("softmax", X, y, classes=4), 10, 1, 12, "k_batch_async", od, 0.05, seed=52, adasync=ada)
    ctx.run(170)
    tr.run(170)
    g, o = ctx.trace(), tr.trace()
    assert o["K"][-1] == 8 and o["K"][0] == 1
    assert_trace_equal(g, o)
    assert np.allclose(g["loss"], o["loss"], rtol=FP32_LOSS_RTOL, atol=1e-6)
    assert rel(ctx.params(), tr.params()) <= FP32_PARAM_TOL
    ctx.close()


def test_stream_read_rate_is_plausible(ssgd, torch_cuda):
    """The plain read kernel behind the 'achievable ceiling' figure: on 1 GiB (more than the last-level cache holds)
    between 1 TB/s and the 8 TB/s the memory is specified for, and an invalid buffer is refused."""
    torch = torch_cuda
    x = torch.ones(256 << 20, dtype=torch.float32, device="cuda")
    rate = ssgd.stream_read_rate(x, passes=5)
    assert 1.0e12 < rate < 8.0e12, rate
    with pytest.raises(ssgd.SsgdError):
        ssgd.stream_read_rate(x[1:], passes=1)          # not 16-byte aligned


# ------------------------------------------------------------------------------- config 2 at its full horizon

def test_config2_softmax_kbatch_sync_full_size(ssgd, oracle, torch_cuda, mixture_full, config2_oracle_run):
    """P=64, m=128, K=16, Pareto(2.5, 1), lr=0.05 on the d=3072 data, J=2000: 25 iterations as single steps with
    the averaged gradient compared (each iteration is 32 tiles of 64 rows in the steady-state kernel), then the
    whole run: schedule, loss trace and the parameters at J against the oracle, whose 2000 iterations (about two
    minutes on one core) run in a thread of their own from the start of this module."""
    torch = torch_cuda
    X, y, Xd, yd = mixture_full
    gd, od = dist_pair(ssgd, oracle, ("pareto", 2.5, 1.0))
    J = 2000
    ctx = ssgd.Context("softmax", Xd, yd, 64, 16, 128, "k_batch_sync", gd, 0.05, seed=0, classes=10)
    tr = oracle.Trainer(oracle.Model("softmax", X, y, classes=10), 64, 16, 128, "k_batch_sync", od, 0.05, seed=0)
    agg = torch.zeros(ctx.nw, device="cuda")
    worst = 0.0
    for j in range(25):
        ctx.step(agg)
        worst = max(worst, rel(agg.cpu().numpy(), tr.step()))
    assert worst <= GRAD_TOL, worst
    assert_trace_equal(ctx.trace(), tr.trace())
    assert rel(ctx.params(), tr.params()) <= FP32_PARAM_TOL
    ctx.run(J - 25)
    full = config2_oracle_run.result()
    assert full.updates == J
    assert_trace_equal(ctx.trace(), full.trace())
    pr = rel(ctx.params(), full.params())
    print(f"config 2: worst per-step gradient error {worst:.3e}, parameter error after {J} iterations {pr:.3e}")
    assert pr <= FP32_PARAM_TOL, pr
    assert np.allclose(ctx.trace()["loss"], full.trace()["loss"], rtol=FP32_LOSS_RTOL, atol=1e-6)
    ctx.close()
