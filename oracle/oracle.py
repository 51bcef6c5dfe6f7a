"""ctypes front end of the CPU oracle (oracle/aet_oracle.c).  TEST INFRASTRUCTURE ONLY.

The C file is compiled twice: REAL=double (the reference every parity test compares
against) and REAL=float (a twin used to see how much plain fp32 rounding moves the
result).  Nothing here is shared with, or imported by, the HIP path.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "aet_oracle.c")
_MAX_LAYERS = 16


class _Layer(C.Structure):
    _fields_ = [("type", C.c_int32), ("cout", C.c_int32), ("k", C.c_int32),
                ("pad", C.c_int32), ("relu", C.c_int32)]


class _Model(C.Structure):
    _fields_ = [("in_c", C.c_int32), ("in_h", C.c_int32), ("in_w", C.c_int32),
                ("n_layers", C.c_int32), ("batch", C.c_int32),
                ("layers", _Layer * _MAX_LAYERS)]


def _lib_path(prec: str) -> str:
    return os.path.join(_HERE, f"libaet_oracle_{prec}.so")


def build(force: bool = True) -> None:
    """Compile both precisions with gcc.  -ffp-contract=off: no fused multiply-add, so
    the arithmetic is exactly what the source says."""
    for prec, real in (("f64", "double"), ("f32", "float")):
        out = _lib_path(prec)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               f"-DREAL={real}", "-o", out, _SRC, "-lm"]
        subprocess.run(cmd, check=True)


_LIBS = {}


def load(prec: str = "f64"):
    if prec in _LIBS:
        return _LIBS[prec]
    path = _lib_path(prec)
    if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_SRC):
        build(force=True)
    lib = C.CDLL(path)
    u64, i64, i32, dbl, vp = C.c_uint64, C.c_int64, C.c_int32, C.c_double, C.c_void_p
    lib.orc_draw.restype = u64
    lib.orc_draw.argtypes = [u64, u64]
    lib.orc_stream.restype = u64
    lib.orc_stream.argtypes = [u64, u64, u64, u64]
    lib.orc_sample_index.restype = i32
    lib.orc_sample_index.argtypes = [u64, i32, i64, i64]
    lib.orc_net_delay.restype = i32
    lib.orc_net_delay.argtypes = [u64, i32, i32, i32, i32]
    lib.orc_threshold.restype = i64
    lib.orc_threshold.argtypes = [i64, i64, i64]
    lib.orc_rounds_needed.restype = i64
    lib.orc_rounds_needed.argtypes = [i64, i64, i64]
    lib.orc_eta.restype = dbl
    lib.orc_eta.argtypes = [dbl, dbl, dbl, i64]
    lib.orc_n_params.restype = i64
    lib.orc_n_params.argtypes = [C.POINTER(_Model)]
    lib.orc_batch_loss_grad.restype = dbl
    lib.orc_batch_loss_grad.argtypes = [C.POINTER(_Model), vp, vp, vp, i32, vp]
    lib.orc_create.restype = vp
    lib.orc_create.argtypes = [C.POINTER(_Model), i32, vp, vp, vp, vp, u64]
    lib.orc_destroy.restype = None
    lib.orc_destroy.argtypes = [vp]
    lib.orc_last_error.restype = C.c_char_p
    lib.orc_last_error.argtypes = [vp]
    lib.orc_run_round.restype = C.c_int
    lib.orc_run_round.argtypes = [vp, i64, i64, i32, dbl, dbl, dbl, vp, vp, i32, i32, u64, i32,
                                  vp, vp, vp]
    lib.orc_server_aggregate.restype = C.c_int
    lib.orc_server_aggregate.argtypes = [vp, dbl, vp, vp, vp]
    lib.orc_set_setup.restype = C.c_int
    lib.orc_set_setup.argtypes = [vp, vp, u64]
    lib.orc_setup_owner.restype = i32
    lib.orc_setup_owner.argtypes = [u64, vp, i32, i64, i64]
    lib.orc_set_topology.restype = C.c_int
    lib.orc_set_topology.argtypes = [vp, vp, vp]
    lib.orc_receive.restype = C.c_int
    lib.orc_receive.argtypes = [vp, dbl, vp, vp, vp]
    lib.orc_all_done.restype = C.c_int
    lib.orc_all_done.argtypes = [vp, i32]
    for name in ("orc_tick", "orc_queue_len", "orc_params", "orc_event_count"):
        getattr(lib, name).restype = i64
        getattr(lib, name).argtypes = [vp]
    lib.orc_get_U.restype = C.c_int
    lib.orc_get_U.argtypes = [vp, i32, i32, vp]
    lib.orc_get_weights.restype = C.c_int
    lib.orc_get_weights.argtypes = [vp, i32, vp]
    lib.orc_set_weights.restype = C.c_int
    lib.orc_set_weights.argtypes = [vp, i32, vp]
    lib.orc_get_round_info.restype = C.c_int
    lib.orc_get_round_info.argtypes = [vp, i32, i32, vp, vp]
    lib.orc_get_events.restype = None
    lib.orc_get_events.argtypes = [vp, vp, vp, vp]
    lib.orc_history.restype = i64
    lib.orc_history.argtypes = [vp, i32]
    lib.orc_real_bytes.restype = C.c_int
    lib.orc_real_bytes.argtypes = []
    lib.orc_set_kink_eps.restype = None
    lib.orc_set_kink_eps.argtypes = [vp, dbl]
    lib.orc_n_tensors.restype = i32
    lib.orc_n_tensors.argtypes = [vp]
    lib.orc_get_round_kinks.restype = C.c_int
    lib.orc_get_round_kinks.argtypes = [vp, i32, i32, vp, vp]
    lib.orc_sample_kinks.restype = i64
    lib.orc_sample_kinks.argtypes = [C.POINTER(_Model), vp, vp, i32, dbl, i64, vp, vp, vp, vp]
    _LIBS[prec] = lib
    return lib


def _c_model(model) -> _Model:
    m = _Model()
    m.in_c, m.in_h, m.in_w = model.in_c, model.in_h, model.in_w
    m.n_layers, m.batch = len(model.layers), model.batch
    for j, L in enumerate(model.layers):
        m.layers[j] = _Layer(L.type, L.cout, L.k, L.pad, L.relu)
    return m


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def batch_loss_grad(model, w: np.ndarray, X: np.ndarray, y: np.ndarray, prec: str = "f64",
                    want_grad: bool = True):
    """Mean loss and mean gradient of one mini-batch at weights w."""
    lib = load(prec)
    dt = np.float64 if prec == "f64" else np.float32
    w = np.ascontiguousarray(w, dtype=dt)
    X = np.ascontiguousarray(X, dtype=np.float32)
    y = np.ascontiguousarray(y, dtype=np.int32)
    g = np.empty_like(w) if want_grad else None
    cm = _c_model(model)
    loss = lib.orc_batch_loss_grad(C.byref(cm), _ptr(w), _ptr(X), _ptr(y), X.shape[0], _ptr(g))
    if loss < 0 and loss in (-1.0, -2.0):
        raise ValueError("oracle rejected the model")
    return loss, g


def sample_kinks(model, w: np.ndarray, x: np.ndarray, label: int, eps: float, cap: int = 4096,
                 prec: str = "f64"):
    """Near-kink decisions of one sample at weights w (see "Kinks" in the C source):
    (events, allow) with events = [(layer, unit, jump vector)], allow per parameter tensor."""
    lib = load(prec)
    dt = np.float64 if prec == "f64" else np.float32
    w = np.ascontiguousarray(w, dtype=dt)
    x = np.ascontiguousarray(x, dtype=np.float32)
    cm = _c_model(model)
    nt = 2 * sum(1 for L in model.layers if L.type != 1)
    lay = np.zeros(cap, dtype=np.int32)
    unit = np.zeros(cap, dtype=np.int64)
    jump = np.zeros((cap, w.size), dtype=dt)
    allow = np.zeros(nt, dtype=np.float64)
    n = int(lib.orc_sample_kinks(C.byref(cm), _ptr(w), _ptr(x), int(label), float(eps), cap,
                                 _ptr(lay), _ptr(unit), _ptr(jump), _ptr(allow)))
    if n < 0:
        raise ValueError("oracle rejected the model")
    m = min(n, cap)
    return [(int(lay[j]), int(unit[j]), jump[j].copy()) for j in range(m)], allow, n


class Oracle:
    """One run of the client/round/server loop on the CPU."""

    def __init__(self, wl, prec: str = "f64", n_clients: Optional[int] = None):
        self.lib = load(prec)
        self.dtype = np.float64 if prec == "f64" else np.float32
        self.wl = wl
        self.n = wl.n_clients if n_clients is None else n_clients
        self._X = [np.ascontiguousarray(x, dtype=np.float32) for x in wl.X[: self.n]]
        self._y = [np.ascontiguousarray(v, dtype=np.int32) for v in wl.y[: self.n]]
        Xp = (C.c_void_p * self.n)(*[x.ctypes.data for x in self._X])
        yp = (C.c_void_p * self.n)(*[v.ctypes.data for v in self._y])
        ns = np.array([x.shape[0] for x in self._X], dtype=np.int64)
        self._w0 = np.ascontiguousarray(wl.w0, dtype=np.float32)
        cm = _c_model(wl.model)
        self.ctx = self.lib.orc_create(C.byref(cm), self.n, Xp, yp, _ptr(ns), _ptr(self._w0),
                                       C.c_uint64(wl.seed))
        if not self.ctx:
            raise ValueError("orc_create failed")
        self.P = int(self.lib.orc_params(self.ctx))
        self._cf = None if wl.compute_factor is None else np.ascontiguousarray(
            wl.compute_factor[: self.n], dtype=np.int32)
        self._st = None if wl.is_straggler is None else np.ascontiguousarray(
            wl.is_straggler[: self.n], dtype=np.uint8)
        self.p2p = False
        if getattr(wl, "topology", None) is not None and self.n == wl.n_clients:
            self.set_topology(*wl.topology)
        if getattr(wl, "setup_weights", None) is not None and self.n == wl.n_clients:
            self.set_setup(wl.setup_weights, wl.setup_seed)

    def close(self):
        if self.ctx:
            self.lib.orc_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != 0:
            raise RuntimeError(self.lib.orc_last_error(self.ctx).decode())

    def run_round(self, rounds: Optional[int] = None, a=None, b=None, d_max=None):
        wl = self.wl
        nf = C.c_int32(0)
        fc = np.zeros(self.n, dtype=np.int32)
        fr = np.zeros(self.n, dtype=np.int32)
        self._check(self.lib.orc_run_round(
            self.ctx, wl.a if a is None else a, wl.b if b is None else b,
            wl.rounds if rounds is None else rounds, wl.eta0, wl.beta, wl.power,
            _ptr(self._cf), _ptr(self._st), wl.delay_min, wl.delay_max,
            C.c_uint64(wl.delay_seed), wl.d_max if d_max is None else d_max,
            C.byref(nf), _ptr(fc), _ptr(fr)))
        return list(zip(fc[: nf.value].tolist(), fr[: nf.value].tolist()))

    def server_aggregate(self, agg_scale: Optional[float] = None):
        na = C.c_int32(0)
        cap = max(1, int(self.lib.orc_queue_len(self.ctx)))
        ac = np.zeros(cap, dtype=np.int32)
        ar = np.zeros(cap, dtype=np.int32)
        self._check(self.lib.orc_server_aggregate(
            self.ctx, self.wl.agg_scale if agg_scale is None else agg_scale,
            C.byref(na), _ptr(ac), _ptr(ar)))
        return list(zip(ac[: na.value].tolist(), ar[: na.value].tolist()))

    def set_setup(self, weights, seed: int):
        """Round lengths from the coin flips of Algorithm 1 (Setup); the workload's
        threshold becomes the global sequence."""
        self._weights = np.ascontiguousarray(weights, dtype=np.uint32)
        assert self._weights.shape[0] == self.n
        self._check(self.lib.orc_set_setup(self.ctx, _ptr(self._weights), C.c_uint64(seed)))

    def set_topology(self, nbr_off, nbr):
        """Peer-to-peer form on the given neighbour lists (CSR)."""
        self._nbr_off = np.ascontiguousarray(nbr_off, dtype=np.int32)
        self._nbr = np.ascontiguousarray(nbr, dtype=np.int32)
        assert self._nbr_off.shape[0] == self.n + 1
        self._check(self.lib.orc_set_topology(self.ctx, _ptr(self._nbr_off), _ptr(self._nbr)))
        self.p2p = True

    def receive(self, scale: Optional[float] = None):
        na = C.c_int32(0)
        cap = max(1, int(self.lib.orc_queue_len(self.ctx)))
        ac = np.zeros(cap, dtype=np.int32)
        ar = np.zeros(cap, dtype=np.int32)
        self._check(self.lib.orc_receive(
            self.ctx, self.wl.agg_scale if scale is None else scale, C.byref(na), _ptr(ac), _ptr(ar)))
        return list(zip(ac[: na.value].tolist(), ar[: na.value].tolist()))

    def exchange(self, scale: Optional[float] = None):
        """The tick's second half: Receive at the neighbours or at the server."""
        return self.receive(scale) if self.p2p else self.server_aggregate(scale)

    def all_done(self, rounds: Optional[int] = None) -> bool:
        return bool(self.lib.orc_all_done(self.ctx, self.wl.rounds if rounds is None else rounds))

    def get_U(self, c: int, k: int) -> np.ndarray:
        out = np.empty(self.P, dtype=self.dtype)
        self._check(self.lib.orc_get_U(self.ctx, c, k, _ptr(out)))
        return out

    def get_weights(self, c: int = -1) -> np.ndarray:
        out = np.empty(self.P, dtype=self.dtype)
        self._check(self.lib.orc_get_weights(self.ctx, c, _ptr(out)))
        return out

    def set_weights(self, c: int, w: np.ndarray):
        w = np.ascontiguousarray(w, dtype=self.dtype)
        assert w.size == self.P
        self._check(self.lib.orc_set_weights(self.ctx, c, _ptr(w)))

    def round_info(self, c: int, k: int) -> dict:
        ints = np.zeros(6, dtype=np.int64)
        dbl = np.zeros(2, dtype=np.float64)
        self._check(self.lib.orc_get_round_info(self.ctx, c, k, _ptr(ints), _ptr(dbl)))
        return dict(s=int(ints[0]), m=int(ints[1]), q0=int(ints[2]), t0=int(ints[3]),
                    start_tick=int(ints[4]), arrival=int(ints[5]), eta=float(dbl[0]),
                    loss=float(dbl[1]))

    def set_kink_eps(self, eps: float):
        """Kink analysis on (eps > 0) or off for the rounds that follow."""
        self.lib.orc_set_kink_eps(self.ctx, float(eps))

    def round_kinks(self, c: int, k: int):
        """(number of near-kink decisions, allowance per parameter tensor) of round k of c."""
        ev = C.c_int64(0)
        allow = np.zeros(int(self.lib.orc_n_tensors(self.ctx)), dtype=np.float64)
        self._check(self.lib.orc_get_round_kinks(self.ctx, c, k, C.byref(ev), _ptr(allow)))
        return ev.value, allow

    def events(self):
        n = int(self.lib.orc_event_count(self.ctx))
        t = np.zeros(max(n, 1), dtype=np.int64)
        c = np.zeros(max(n, 1), dtype=np.int32)
        k = np.zeros(max(n, 1), dtype=np.int32)
        self.lib.orc_get_events(self.ctx, _ptr(t), _ptr(c), _ptr(k))
        return list(zip(t[:n].tolist(), c[:n].tolist(), k[:n].tolist()))

    def history(self, c: int) -> int:
        return int(self.lib.orc_history(self.ctx, c))

    @property
    def tick(self) -> int:
        return int(self.lib.orc_tick(self.ctx))

    def run_all(self, rounds: Optional[int] = None, max_ticks: int = 100000):
        """Tick until every client has done its rounds and the queue has drained."""
        R = self.wl.rounds if rounds is None else rounds
        ticks = 0
        while not self.all_done(R):
            self.run_round(R)
            self.exchange()
            ticks += 1
            if ticks > max_ticks:
                raise RuntimeError("oracle did not finish")
        return ticks

    def sample_index(self, c: int, q: int, n_samples: int) -> int:
        return int(self.lib.orc_sample_index(C.c_uint64(self.wl.seed), c, q, n_samples))
