"""CPU oracle (test infrastructure): ctypes view of ``ssgd_oracle.c``.

The C file is a plain sequential restatement of the paper's update rules
(Sec. 2.2), delay model (Sec. 3.1), AdaSync (Sec. 6) and of the runtime
simulation behind Fig. 6.  Only tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the GPU library never does.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ssgd_oracle.c")
_LIB = os.path.join(_HERE, "libssgd_oracle.so")

LSQ, SOFTMAX, MLP2 = 0, 1, 2
K_SYNC, K_BATCH_SYNC, K_ASYNC, K_BATCH_ASYNC = 0, 1, 2, 3
EXP, SHIFTED_EXP, PARETO, TABLE = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
             _SRC, "-o", _LIB, "-lm"])
    return _LIB


class _Dist(C.Structure):
    _fields_ = [("kind", C.c_int32), ("shift", C.c_double), ("rate", C.c_double),
                ("alpha", C.c_double), ("scale", C.c_double),
                ("table", C.POINTER(C.c_float)), ("table_len", C.c_int64)]


class _Model(C.Structure):
    _fields_ = [("kind", C.c_int32), ("d", C.c_int32), ("classes", C.c_int32),
                ("hidden", C.c_int32), ("bf16", C.c_int32),
                ("X", C.c_void_p), ("y", C.c_void_p), ("N", C.c_int64)]


class _Ada(C.Structure):
    _fields_ = [("mode", C.c_int32), ("K0", C.c_int32), ("Kmax", C.c_int32), ("window", C.c_int32),
                ("rel_tol", C.c_double), ("interval_t", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.orc_uniform.restype = C.c_float
        L.orc_uniform.argtypes = [C.c_uint32]
        L.orc_neg_ln.restype = C.c_float
        L.orc_neg_ln.argtypes = [C.c_float]
        L.orc_exp_pos.restype = C.c_float
        L.orc_exp_pos.argtypes = [C.c_float]
        L.orc_round_bf16.restype = C.c_float
        L.orc_round_bf16.argtypes = [C.c_float]
        L.orc_delay_from_bits.restype = C.c_float
        L.orc_delay_from_bits.argtypes = [C.POINTER(_Dist), C.c_uint32]
        L.orc_delays_from_bits.argtypes = [C.POINTER(_Dist), C.c_void_p, C.c_int64, C.c_void_p]
        L.orc_delay.restype = C.c_float
        L.orc_delay.argtypes = [C.POINTER(_Dist), C.c_uint64, C.c_uint32, C.c_int32, C.c_int32,
                                C.c_uint32, C.c_uint32, C.c_uint32]
        L.orc_batch_index.restype = C.c_uint32
        L.orc_batch_index.argtypes = [C.c_uint64] + [C.c_uint32] * 6
        L.orc_param_count.restype = C.c_int64
        L.orc_param_count.argtypes = [C.POINTER(_Model)]
        L.orc_minibatch_grad.restype = C.c_double
        L.orc_minibatch_grad.argtypes = [C.POINTER(_Model), C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        L.orc_full_loss.restype = C.c_double
        L.orc_full_loss.argtypes = [C.POINTER(_Model), C.c_void_p]
        L.orc_full_grad.argtypes = [C.POINTER(_Model), C.c_void_p, C.c_void_p]
        L.orc_init_params.argtypes = [C.POINTER(_Model), C.c_uint64, C.c_void_p]
        L.orc_create.restype = C.c_void_p
        L.orc_create.argtypes = [C.POINTER(_Model), C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                 C.POINTER(_Dist), C.c_double, C.c_uint64, C.c_uint32, C.POINTER(_Ada)]
        L.orc_destroy.argtypes = [C.c_void_p]
        L.orc_step.argtypes = [C.c_void_p, C.c_void_p]
        L.orc_run.argtypes = [C.c_void_p, C.c_int64]
        L.orc_updates_done.restype = C.c_int64
        L.orc_updates_done.argtypes = [C.c_void_p]
        L.orc_current_K.argtypes = [C.c_void_p]
        L.orc_trace_width.argtypes = [C.c_void_p]
        L.orc_clock.restype = C.c_double
        L.orc_clock.argtypes = [C.c_void_p]
        L.orc_get_params.argtypes = [C.c_void_p, C.c_void_p]
        L.orc_set_params.argtypes = [C.c_void_p, C.c_void_p]
        L.orc_force_K.argtypes = [C.c_void_p, C.c_int32]
        L.orc_get_trace.argtypes = [C.c_void_p, C.c_int64, C.c_int64] + [C.c_void_p] * 6
        L.orc_get_workers.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_runtime_mc.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(_Dist),
                                     C.c_int64, C.c_int64, C.c_int32, C.c_uint64,
                                     C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return out


class Dist:
    """Delay distribution: ('exp', rate) | ('shifted_exp', shift, rate) |
    ('pareto', alpha, scale) | ('table', array)."""

    def __init__(self, kind, *args):
        self.spec = (kind,) + tuple(args)
        self._keep = None
        d = _Dist()
        d.shift = 0.0
        d.rate = 1.0
        d.alpha = 1.0
        d.scale = 1.0
        d.table = None
        d.table_len = 0
        if kind == "exp":
            d.kind, d.rate = EXP, float(args[0])
        elif kind == "shifted_exp":
            d.kind, d.shift, d.rate = SHIFTED_EXP, float(args[0]), float(args[1])
        elif kind == "pareto":
            d.kind, d.alpha, d.scale = PARETO, float(args[0]), float(args[1])
        elif kind == "table":
            self._keep = np.ascontiguousarray(args[0], dtype=np.float32)
            d.kind = TABLE
            d.table = self._keep.ctypes.data_as(C.POINTER(C.c_float))
            d.table_len = self._keep.size
        else:
            raise ValueError(kind)
        self.c = d

    def from_bits(self, bits):
        bits = np.ascontiguousarray(np.atleast_1d(bits), dtype=np.uint32)
        out = np.zeros(bits.size, dtype=np.float32)
        lib().orc_delays_from_bits(C.byref(self.c), bits.ctypes.data, bits.size, out.ctypes.data)
        return out


def delay(dist: Dist, seed, replica, P, table_ord, worker, ordinal, version):
    return np.float32(lib().orc_delay(C.byref(dist.c), seed, replica, P, table_ord, worker, ordinal, version))


def batch_indices(seed, replica, worker, ordinal, version, m, N):
    f = lib().orc_batch_index
    return np.array([f(seed, replica, worker, ordinal, version, s, N) for s in range(m)], dtype=np.uint32)


class Model:
    def __init__(self, kind, X, y, classes=1, hidden=0, bf16=0):
        self.X = np.ascontiguousarray(X, dtype=np.float32)
        self.kind = {"lsq": LSQ, "softmax": SOFTMAX, "mlp2": MLP2}[kind]
        self.y = np.ascontiguousarray(y, dtype=np.float32 if self.kind == LSQ else np.int32)
        m = _Model()
        m.kind = self.kind
        m.N, m.d = self.X.shape
        m.classes, m.hidden, m.bf16 = classes, hidden, bf16
        m.X = self.X.ctypes.data
        m.y = self.y.ctypes.data
        self.c = m
        self.nw = int(lib().orc_param_count(C.byref(m)))

    def init_params(self, seed=0):
        w = np.zeros(self.nw, dtype=np.float32)
        lib().orc_init_params(C.byref(self.c), seed, w.ctypes.data)
        return w

    def minibatch_grad(self, w, idx):
        w = np.ascontiguousarray(w, dtype=np.float32)
        idx = np.ascontiguousarray(idx, dtype=np.uint32)
        g = np.zeros(self.nw, dtype=np.float64)
        loss = lib().orc_minibatch_grad(C.byref(self.c), w.ctypes.data, idx.ctypes.data, idx.size, g.ctypes.data)
        return g, float(loss)

    def full_loss(self, w):
        w = np.ascontiguousarray(w, dtype=np.float32)
        return float(lib().orc_full_loss(C.byref(self.c), w.ctypes.data))

    def full_grad(self, w):
        """Gradient of the objective over the whole data set (Eq. (1)), fp64."""
        w = np.ascontiguousarray(w, dtype=np.float32)
        out = np.zeros(self.nw, dtype=np.float64)
        lib().orc_full_grad(C.byref(self.c), w.ctypes.data, out.ctypes.data)
        return out


_VARIANTS = {"k_sync": K_SYNC, "k_batch_sync": K_BATCH_SYNC, "k_async": K_ASYNC,
             "k_batch_async": K_BATCH_ASYNC}


class Trainer:
    """One replica of the parameter-server simulation."""

    def __init__(self, model: Model, P, K, m, variant, dist: Dist, lr, seed=0, replica=0, adasync=None):
        self.model, self.dist = model, dist
        ada = None
        if adasync is not None:
            a = _Ada()
            a.mode = adasync.get("mode", 0)
            a.K0 = adasync.get("K0", K)
            a.Kmax = adasync.get("Kmax", K)
            a.window = adasync.get("window", 200)
            a.rel_tol = adasync.get("rel_tol", 0.01)
            a.interval_t = adasync.get("interval_t", 1.0)
            ada = C.byref(a)
        self.h = lib().orc_create(C.byref(model.c), P, K, m, _VARIANTS[variant], C.byref(dist.c),
                                  float(lr), seed, replica, ada)
        if not self.h:
            raise ValueError("orc_create rejected the arguments")
        self.P = P
        self.width = lib().orc_trace_width(self.h)

    def __del__(self):
        if getattr(self, "h", None):
            lib().orc_destroy(self.h)
            self.h = None

    def step(self, want_grad=True):
        g = np.zeros(self.model.nw, dtype=np.float64) if want_grad else None
        lib().orc_step(self.h, g.ctypes.data if want_grad else None)
        return g

    def run(self, J):
        lib().orc_run(self.h, J)

    @property
    def updates(self):
        return int(lib().orc_updates_done(self.h))

    @property
    def K(self):
        return int(lib().orc_current_K(self.h))

    @property
    def clock(self):
        return float(lib().orc_clock(self.h))

    def force_K(self, K):
        lib().orc_force_K(self.h, K)

    def params(self):
        w = np.zeros(self.model.nw, dtype=np.float32)
        lib().orc_get_params(self.h, w.ctypes.data)
        return w

    def set_params(self, w):
        w = np.ascontiguousarray(w, dtype=np.float32)
        lib().orc_set_params(self.h, w.ctypes.data)

    def workers(self):
        tau = np.zeros(self.P, dtype=np.int64)
        fin = np.zeros(self.P, dtype=np.float64)
        lib().orc_get_workers(self.h, tau.ctypes.data, fin.ctypes.data)
        return tau, fin

    def trace(self, start=0, n=None):
        n = self.updates - start if n is None else n
        W = self.width
        t = np.zeros(n, dtype=np.float64)
        loss = np.zeros(n, dtype=np.float32)
        K = np.zeros(n, dtype=np.int32)
        sel = np.zeros((n, W), dtype=np.int32)
        stale = np.zeros((n, W), dtype=np.int32)
        ordn = np.zeros((n, W), dtype=np.int32)
        rc = lib().orc_get_trace(self.h, start, n, t.ctypes.data, loss.ctypes.data, K.ctypes.data,
                                 sel.ctypes.data, stale.ctypes.data, ordn.ctypes.data)
        if rc:
            raise IndexError("trace range")
        return dict(t=t, loss=loss, K=K, sel=sel, staleness=stale, ordinal=ordn)


def runtime_mc(variant, P, Kmin, Kmax, dist: Dist, trials, chain_len, seed=0, trial0=0, per_trial=False):
    """Sums and sums of squares of T_l per (K, l); optionally every trial's values."""
    nK = Kmax - Kmin + 1
    s = np.zeros((nK, chain_len), dtype=np.float64)
    s2 = np.zeros((nK, chain_len), dtype=np.float64)
    pt = np.zeros((trials, nK, chain_len), dtype=np.float64) if per_trial else None
    rc = lib().orc_runtime_mc(_VARIANTS[variant], P, Kmin, Kmax, C.byref(dist.c), trial0, trials,
                              chain_len, seed, s.ctypes.data, s2.ctypes.data,
                              pt.ctypes.data if per_trial else None)
    if rc:
        raise ValueError("orc_runtime_mc rejected the arguments")
    mean = s / trials
    var = (s2 - s * s / trials) / (trials - 1) if trials > 1 else np.zeros_like(s)
    return dict(mean=mean, var=var, sum=s, sumsq=s2, per_trial=pt)
