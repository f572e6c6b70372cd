"""ctypes binding of libssgd.so: the same names as include/ssgd.h, argument
marshalling only.  PyTorch supplies device memory and the stream handle."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libssgd.so")

LSQ, SOFTMAX, MLP2 = 0, 1, 2
K_SYNC, K_BATCH_SYNC, K_ASYNC, K_BATCH_ASYNC = 0, 1, 2, 3
EXP, SHIFTED_EXP, PARETO, TABLE = 0, 1, 2, 3
OK, EINVAL, ENOMEM, EDEVICE, ESTATE = 0, 1, 2, 3, 4
_VARIANTS = {"k_sync": K_SYNC, "k_batch_sync": K_BATCH_SYNC, "k_async": K_ASYNC, "k_batch_async": K_BATCH_ASYNC}
_KINDS = {"lsq": LSQ, "softmax": SOFTMAX, "mlp2": MLP2}

EXPORTS = [
    "ssgd_create", "ssgd_run", "ssgd_reserve_trace", "ssgd_step", "ssgd_param_count", "ssgd_updates_done", "ssgd_current_K",
    "ssgd_trace_width", "ssgd_get_trace", "ssgd_get_params", "ssgd_set_params", "ssgd_force_K",
    "ssgd_get_workers", "ssgd_state_bytes", "ssgd_get_state", "ssgd_set_state", "ssgd_full_loss",
    "ssgd_full_gradient", "ssgd_full_gradient_static",
    "ssgd_runtime_mc", "ssgd_debug_delays", "ssgd_debug_batch", "ssgd_stream_read_rate", "ssgd_last_error",
    "ssgd_last_kernel_ms",
    "ssgd_destroy",
]


class SsgdError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"ssgd status {status}: {msg}")
        self.status = status


class DelayDist(C.Structure):
    _fields_ = [("kind", C.c_int32), ("shift", C.c_double), ("rate", C.c_double), ("alpha", C.c_double),
                ("scale", C.c_double), ("table", C.POINTER(C.c_float)), ("table_len", C.c_int64)]


class ModelDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("d", C.c_int32), ("classes", C.c_int32), ("hidden", C.c_int32),
                ("bf16", C.c_int32), ("X", C.c_void_p), ("y", C.c_void_p), ("N", C.c_int64)]


class AdaSync(C.Structure):
    _fields_ = [("mode", C.c_int32), ("K0", C.c_int32), ("Kmax", C.c_int32), ("window", C.c_int32),
                ("rel_tol", C.c_double), ("interval_t", C.c_double)]


_lib = None


def _preload_hip_runtime():
    """PyTorch ships its own HIP runtime; the library must bind to that copy (one runtime per
    process), so it is loaded first, by path, whether or not torch has been imported yet."""
    import importlib.util
    spec = importlib.util.find_spec("torch")
    if spec is not None and spec.origin:
        cand = os.path.join(os.path.dirname(spec.origin), "lib", "libamdhip64.so")
        if os.path.exists(cand):
            C.CDLL(cand, mode=C.RTLD_GLOBAL)


def lib():
    """Load the built library; there is no fallback when it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is not built: run `python -m paper_2003_10579_amd.build`")
        _preload_hip_runtime()
        L = C.CDLL(_LIB_PATH)
        L.ssgd_create.argtypes = [C.POINTER(ModelDesc), C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                  C.POINTER(DelayDist), C.c_double, C.c_uint64, C.c_int32, C.POINTER(AdaSync),
                                  C.c_void_p, C.POINTER(C.c_void_p)]
        L.ssgd_run.argtypes = [C.c_void_p, C.c_int64]
        L.ssgd_reserve_trace.argtypes = [C.c_void_p, C.c_int64]
        L.ssgd_step.argtypes = [C.c_void_p, C.c_void_p]
        L.ssgd_param_count.restype = C.c_int64
        L.ssgd_param_count.argtypes = [C.c_void_p]
        L.ssgd_updates_done.restype = C.c_int64
        L.ssgd_updates_done.argtypes = [C.c_void_p]
        L.ssgd_current_K.argtypes = [C.c_void_p, C.c_int32]
        L.ssgd_trace_width.argtypes = [C.c_void_p]
        L.ssgd_get_trace.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int64] + [C.c_void_p] * 6
        L.ssgd_get_params.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        L.ssgd_set_params.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        L.ssgd_force_K.argtypes = [C.c_void_p, C.c_int32]
        L.ssgd_full_loss.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_double)]
        L.ssgd_full_gradient.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        L.ssgd_full_gradient_static.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        L.ssgd_get_workers.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.ssgd_state_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_int64)]
        L.ssgd_get_state.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        L.ssgd_set_state.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        L.ssgd_runtime_mc.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(DelayDist), C.c_int64,
                                      C.c_int64, C.c_int32, C.c_uint64, C.c_void_p] + [C.c_void_p] * 5
        L.ssgd_debug_delays.argtypes = [C.POINTER(DelayDist), C.c_void_p, C.c_int64, C.c_void_p]
        L.ssgd_debug_batch.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_int32,
                                       C.c_int64, C.c_void_p]
        L.ssgd_stream_read_rate.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.POINTER(C.c_double)]
        L.ssgd_last_error.restype = C.c_char_p
        L.ssgd_last_error.argtypes = [C.c_void_p]
        L.ssgd_last_kernel_ms.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.ssgd_destroy.argtypes = [C.c_void_p]
        _lib = L
    return _lib


def _check(status, ctx=None):
    if status != OK:
        raise SsgdError(status, (lib().ssgd_last_error(ctx) or b"").decode())


def delay_dist(kind, *args):
    """('exp', rate) | ('shifted_exp', shift, rate) | ('pareto', alpha, scale) | ('table', host array)."""
    d = DelayDist()
    d.shift, d.rate, d.alpha, d.scale, d.table, d.table_len = 0.0, 1.0, 1.0, 1.0, None, 0
    keep = None
    if kind == "exp":
        d.kind, d.rate = EXP, float(args[0])
    elif kind == "shifted_exp":
        d.kind, d.shift, d.rate = SHIFTED_EXP, float(args[0]), float(args[1])
    elif kind == "pareto":
        d.kind, d.alpha, d.scale = PARETO, float(args[0]), float(args[1])
    elif kind == "table":
        keep = np.ascontiguousarray(args[0], dtype=np.float32)
        d.kind, d.table, d.table_len = TABLE, keep.ctypes.data_as(C.POINTER(C.c_float)), keep.size
    else:
        raise ValueError(kind)
    d._keep = keep
    return d


class Context:
    """ssgd_ctx with the device tensors it borrows kept alive."""

    def __init__(self, kind, X, y, P, K, m, variant, dist, lr, seed=0, replicas=1, classes=1, hidden=0, bf16=0,
                 adasync=None, stream=None):
        import torch
        assert X.is_cuda and X.dtype == torch.float32 and X.is_contiguous()
        assert y.is_cuda and y.is_contiguous()
        self._X, self._y, self._dist = X, y, dist
        md = ModelDesc()
        md.kind = _KINDS[kind]
        md.N, md.d = X.shape
        md.classes, md.hidden, md.bf16 = classes, hidden, bf16
        md.X, md.y = X.data_ptr(), y.data_ptr()
        ada = None
        if adasync is not None:
            a = AdaSync()
            a.mode = adasync.get("mode", 0)
            a.K0 = adasync.get("K0", K)
            a.Kmax = adasync.get("Kmax", K)
            a.window = adasync.get("window", 200)
            a.rel_tol = adasync.get("rel_tol", 0.01)
            a.interval_t = adasync.get("interval_t", 1.0)
            ada = C.byref(a)
        if stream is None:
            stream = torch.cuda.current_stream(X.device).cuda_stream
        self.stream = stream
        h = C.c_void_p()
        with torch.cuda.device(X.device):
            _check(lib().ssgd_create(C.byref(md), P, K, m, _VARIANTS[variant], C.byref(dist), float(lr), seed,
                                     replicas, ada, C.c_void_p(stream), C.byref(h)))
        self.h = h
        self.P, self.replicas = P, replicas
        self.nw = int(lib().ssgd_param_count(h))
        self.width = int(lib().ssgd_trace_width(h))

    def close(self):
        if getattr(self, "h", None):
            lib().ssgd_destroy(self.h)
            self.h = None

    def __del__(self):
        self.close()

    def run(self, J):
        _check(lib().ssgd_run(self.h, J), self.h)

    def reserve_trace(self, updates):
        _check(lib().ssgd_reserve_trace(self.h, updates), self.h)

    def step(self, agg_out=None):
        _check(lib().ssgd_step(self.h, agg_out.data_ptr() if agg_out is not None else None), self.h)

    @property
    def updates(self):
        return int(lib().ssgd_updates_done(self.h))

    def current_K(self, replica=0):
        return int(lib().ssgd_current_K(self.h, replica))

    def force_K(self, K):
        _check(lib().ssgd_force_K(self.h, K), self.h)

    def full_loss(self, replica=0):
        v = C.c_double()
        _check(lib().ssgd_full_loss(self.h, replica, C.byref(v)), self.h)
        return v.value

    def full_gradient(self, replica=0):
        g = np.zeros(self.nw, dtype=np.float32)
        _check(lib().ssgd_full_gradient(self.h, replica, g.ctypes.data), self.h)
        return g

    def full_gradient_static(self, out, replica=0):
        """Same gradient into `out` (a device tensor of |w| floats), through the library's static scratch array:
        nothing is allocated, nothing is awaited (the work is enqueued on the context's stream)."""
        assert out.is_cuda and out.is_contiguous() and out.numel() >= self.nw and out.element_size() == 4
        _check(lib().ssgd_full_gradient_static(self.h, replica, out.data_ptr()), self.h)

    def workers(self, replica=0):
        tau = np.zeros(self.P, dtype=np.int32)
        ordn = np.zeros(self.P, dtype=np.int32)
        finish = np.zeros(self.P, dtype=np.float64)
        _check(lib().ssgd_get_workers(self.h, replica, tau.ctypes.data, ordn.ctypes.data, finish.ctypes.data), self.h)
        return dict(tau=tau, ordinal=ordn, finish=finish)

    def get_state(self):
        n = C.c_int64()
        _check(lib().ssgd_state_bytes(self.h, C.byref(n)), self.h)
        buf = np.zeros(n.value, dtype=np.uint8)
        _check(lib().ssgd_get_state(self.h, buf.ctypes.data, n.value), self.h)
        return buf

    def set_state(self, buf):
        buf = np.ascontiguousarray(buf, dtype=np.uint8)
        _check(lib().ssgd_set_state(self.h, buf.ctypes.data, buf.size), self.h)

    def params(self, replica=0):
        w = np.zeros(self.nw, dtype=np.float32)
        _check(lib().ssgd_get_params(self.h, replica, w.ctypes.data), self.h)
        return w

    def set_params(self, w, replica=0):
        w = np.ascontiguousarray(w, dtype=np.float32)
        assert w.size == self.nw
        _check(lib().ssgd_set_params(self.h, replica, w.ctypes.data), self.h)

    def trace(self, replica=0, start=0, n=None):
        n = self.updates - start if n is None else n
        W = self.width
        t = np.zeros(n, dtype=np.float64)
        loss = np.zeros(n, dtype=np.float32)
        K = np.zeros(n, dtype=np.int32)
        sel = np.zeros((n, W), dtype=np.int32)
        stale = np.zeros((n, W), dtype=np.int32)
        ordn = np.zeros((n, W), dtype=np.int32)
        _check(lib().ssgd_get_trace(self.h, replica, start, n, t.ctypes.data, loss.ctypes.data, K.ctypes.data,
                                    sel.ctypes.data, stale.ctypes.data, ordn.ctypes.data), self.h)
        return dict(t=t, loss=loss, K=K, sel=sel, staleness=stale, ordinal=ordn)

    def last_kernel_ms(self):
        ms, n = C.c_double(), C.c_int64()
        lib().ssgd_last_kernel_ms(self.h, C.byref(ms), C.byref(n))
        return ms.value, n.value


def runtime_mc(variant, P, Kmin, Kmax, dist, trials, chain_len, seed=0, trial0=0, per_trial=False, stream=None):
    nK = Kmax - Kmin + 1
    mean = np.zeros((nK, chain_len)); var = np.zeros((nK, chain_len))
    s = np.zeros((nK, chain_len)); s2 = np.zeros((nK, chain_len))
    pt = np.zeros((trials, nK, chain_len)) if per_trial else None
    _check(lib().ssgd_runtime_mc(_VARIANTS[variant], P, Kmin, Kmax, C.byref(dist), trial0, trials, chain_len, seed,
                                 C.c_void_p(stream) if stream else None, mean.ctypes.data, var.ctypes.data,
                                 s.ctypes.data, s2.ctypes.data, pt.ctypes.data if per_trial else None))
    return dict(mean=mean, var=var, sum=s, sumsq=s2, per_trial=pt)


def debug_delays(dist, bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint32)
    out = np.zeros(bits.size, dtype=np.float32)
    _check(lib().ssgd_debug_delays(C.byref(dist), bits.ctypes.data, bits.size, out.ctypes.data))
    return out


def stream_read_rate(tensor, passes=10, stream=None):
    """Bytes per second of a plain streaming read of a device tensor (the achievable HBM ceiling)."""
    import torch
    handle = (stream or torch.cuda.current_stream()).cuda_stream
    out = C.c_double(0.0)
    _check(lib().ssgd_stream_read_rate(C.c_void_p(tensor.data_ptr()), tensor.numel() * tensor.element_size(), passes,
                                       C.c_void_p(handle), C.byref(out)))
    return out.value


def debug_batch(seed, replica, worker, ordinal, version, m, N):
    out = np.zeros(m, dtype=np.uint32)
    _check(lib().ssgd_debug_batch(seed, replica, worker, ordinal, version, m, N, out.ctypes.data))
    return out
