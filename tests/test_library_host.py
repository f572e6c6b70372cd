"""Host-side checks that need no GPU: the built library loads, exports every symbol the header
declares, and rejects invalid arguments before it touches the device."""
import ctypes as C
import os
import re

import pytest

from paper_2003_10579_amd import ssgd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(ssgd._LIB_PATH):
        from paper_2003_10579_amd import build
        build.build()
    return ssgd.lib()


def test_exports_every_declared_symbol(L):
    header = open(os.path.join(ROOT, "include", "ssgd.h")).read()
    declared = set(re.findall(r"\b(ssgd_[a-z_A-Z0-9]+)\s*\(", header))
    assert declared == set(ssgd.EXPORTS)
    for name in declared:
        assert getattr(L, name) is not None


def test_exports_nothing_but_the_c_abi(L):
    import shutil
    import subprocess
    if shutil.which("nm") is None:
        pytest.skip("nm not available")
    out = subprocess.run(["nm", "-D", "--defined-only", ssgd._LIB_PATH], capture_output=True, text=True, check=True).stdout
    # functions defined by the library itself ("T"); weak instantiations of standard-library templates do not count
    defined = {line.split()[-1] for line in out.splitlines() if len(line.split()) >= 3 and line.split()[-2] == "T"}
    assert defined == set(ssgd.EXPORTS), defined ^ set(ssgd.EXPORTS)


def _model(kind=ssgd.SOFTMAX, d=8, classes=3, X=0x1000, y=0x1000, N=10, hidden=0, bf16=0):
    m = ssgd.ModelDesc()
    m.kind, m.d, m.classes, m.hidden, m.bf16, m.X, m.y, m.N = kind, d, classes, hidden, bf16, X, y, N
    return m


@pytest.mark.parametrize("case", [
    dict(K=0), dict(K=5, P=4), dict(P=0), dict(P=257), dict(m=0), dict(replicas=0), dict(variant=7),
    dict(variant=ssgd.K_BATCH_ASYNC, K=65, P=70), dict(dist=("exp", 0.0)), dict(dist=("pareto", -1.0, 1.0)),
    dict(dist=("shifted_exp", 0.5, -2.0)), dict(model=dict(X=None)), dict(model=dict(N=0)),
    dict(model=dict(classes=17)), dict(model=dict(kind=ssgd.LSQ, bf16=1)), dict(model=dict(kind=9)),
    dict(model=dict(kind=ssgd.MLP2, hidden=100)), dict(ada=dict(mode=1, K0=2, Kmax=1, window=10)),
    # the two-layer network: every limit the header states, refused before anything is allocated
    dict(model=dict(kind=ssgd.MLP2, d=128, hidden=128, classes=4, bf16=0)),      # fp32 operands are not built
    dict(model=dict(kind=ssgd.MLP2, d=128, hidden=192, classes=4, bf16=1)),      # hidden % 128
    dict(model=dict(kind=ssgd.MLP2, d=96, hidden=128, classes=4, bf16=1)),       # d % 128
    dict(model=dict(kind=ssgd.MLP2, d=128, hidden=128, classes=4, bf16=1), m=65),
    dict(model=dict(kind=ssgd.MLP2, d=128, hidden=128, classes=4, bf16=1), replicas=2,
         ada=dict(mode=2, K0=2, Kmax=4, window=0, interval_t=1.0)),   # the paper's rules run one replica
    dict(model=dict(kind=ssgd.MLP2, d=128, hidden=128, classes=17, bf16=1)),
    dict(ada=dict(mode=2, K0=2, Kmax=4, window=0, interval_t=0.0)),
])
def test_create_rejects_invalid_arguments(L, case):
    md = _model(**case.get("model", {}))
    d = ssgd.delay_dist(*case.get("dist", ("exp", 1.0)))
    ada = None
    if "ada" in case:
        a = ssgd.AdaSync()
        a.mode, a.K0, a.Kmax, a.window = (case["ada"][k] for k in ("mode", "K0", "Kmax", "window"))
        a.rel_tol, a.interval_t = 0.01, case["ada"].get("interval_t", 1.0)
        ada = C.byref(a)
    h = C.c_void_p(0x1234)
    st = L.ssgd_create(C.byref(md), case.get("P", 4), case.get("K", 2), case.get("m", 4),
                       case.get("variant", ssgd.K_SYNC), C.byref(d), 0.1, 0, case.get("replicas", 1), ada, None,
                       C.byref(h))
    assert st == ssgd.EINVAL
    assert h.value == 0x1234                      # *out untouched
    assert len(L.ssgd_last_error(None)) > 0


def test_null_context_calls_are_errors(L):
    assert L.ssgd_run(None, 1) == ssgd.EINVAL
    assert L.ssgd_step(None, None) == ssgd.EINVAL
    assert L.ssgd_param_count(None) == -1
    L.ssgd_destroy(None)


def test_runtime_mc_rejects_invalid_arguments(L):
    d = ssgd.delay_dist("exp", 1.0)
    args = lambda **k: (k.get("variant", ssgd.K_ASYNC), k.get("P", 8), k.get("Kmin", 1), k.get("Kmax", 8), C.byref(d),
                        0, k.get("trials", 10), k.get("chain", 2), 0, None, None, None, None, None, None)
    for bad in (dict(P=0), dict(P=300), dict(Kmin=0), dict(Kmax=9), dict(trials=0), dict(chain=0),
                dict(variant=7), dict(Kmax=128, P=128, chain=5000),
                dict(variant=ssgd.K_BATCH_ASYNC, Kmax=128, P=128, chain=64)):
        assert L.ssgd_runtime_mc(*args(**bad)) == ssgd.EINVAL


def test_state_entry_points_reject_null_arguments(L):
    n = C.c_int64(0)
    buf = (C.c_ubyte * 16)()
    assert L.ssgd_state_bytes(None, C.byref(n)) == ssgd.EINVAL
    assert L.ssgd_get_state(None, buf, 16) == ssgd.EINVAL
    assert L.ssgd_set_state(None, buf, 16) == ssgd.EINVAL
    assert L.ssgd_get_workers(None, 0, None, None, None) == ssgd.EINVAL
