"""Thin ctypes binding of libaet_sgd.so: argument marshalling only.  Every step of the
AET-SGD hot path runs in the library's HIP kernels; PyTorch supplies device memory
(shards, workspace) and the stream handle.  There is no CPU fallback: a missing or
unloadable library is an error."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import build as _build

AET_OK, AET_EINVAL, AET_ENOMEM, AET_EHIP, AET_ESTATE = 0, -1, -2, -3, -4
AET_CONV, AET_POOL, AET_DENSE = 0, 1, 2
AET_MAX_LAYERS = 16

EXPORTS = [
    "aet_n_params", "aet_workspace_bytes", "aet_init", "aet_run_round", "aet_server_aggregate",
    "aet_get_U", "aet_get_weights", "aet_get_round_info", "aet_debug_sample_indices",
    "aet_all_done", "aet_tick", "aet_history", "aet_inflight", "aet_synchronize",
    "aet_last_error", "aet_destroy", "aet_reset", "aet_profile_families",
    "aet_profile_family_name", "aet_profile_enable", "aet_profile_read", "aet_run_ticks",
    "aet_topology_workspace_bytes", "aet_set_topology", "aet_receive", "aet_set_setup",
    "aet_set_weights", "aet_init_static", "aet_test_select_kernels",
]


class aet_layer(C.Structure):
    _fields_ = [("type", C.c_int32), ("cout", C.c_int32), ("k", C.c_int32), ("pad", C.c_int32),
                ("relu", C.c_int32)]


class aet_model_desc(C.Structure):
    _fields_ = [("in_c", C.c_int32), ("in_h", C.c_int32), ("in_w", C.c_int32),
                ("n_layers", C.c_int32), ("batch", C.c_int32),
                ("layers", aet_layer * AET_MAX_LAYERS)]


class aet_shard(C.Structure):
    _fields_ = [("X", C.c_void_p), ("y", C.c_void_p), ("n_samples", C.c_int64)]


class aet_threshold(C.Structure):
    _fields_ = [("a", C.c_int64), ("b", C.c_int64), ("rounds", C.c_int32)]


class aet_eta(C.Structure):
    _fields_ = [("eta0", C.c_double), ("beta", C.c_double), ("power", C.c_double)]


class aet_delay(C.Structure):
    _fields_ = [("compute_factor", C.c_void_p), ("is_straggler", C.c_void_p),
                ("delay_min", C.c_int32), ("delay_max", C.c_int32), ("seed", C.c_uint64),
                ("d_max", C.c_int32)]


class AetError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"aet status {status}: {msg}")
        self.status = status


_LIB = None


def load_library():
    """Load the in-tree library (building it only if it has never been built)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = _build.LIB
    if not os.path.exists(path):
        _build.build(force=True)
    lib = C.CDLL(path)
    vp, i32, i64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
    lib.aet_n_params.restype = i64
    lib.aet_n_params.argtypes = [C.POINTER(aet_model_desc)]
    lib.aet_workspace_bytes.restype = C.c_size_t
    lib.aet_workspace_bytes.argtypes = [C.POINTER(aet_model_desc), i32, i32, i32]
    lib.aet_init.restype = C.c_int
    lib.aet_init.argtypes = [C.POINTER(vp), C.POINTER(aet_model_desc), i32, C.POINTER(aet_shard),
                             vp, u64, vp, C.c_size_t, i32, i32, vp]
    lib.aet_init_static.restype = C.c_int
    lib.aet_init_static.argtypes = [C.POINTER(vp), C.POINTER(aet_model_desc), i32, C.POINTER(aet_shard),
                                    vp, u64, i32, i32, vp]
    lib.aet_run_round.restype = C.c_int
    lib.aet_run_round.argtypes = [vp, C.POINTER(aet_threshold), C.POINTER(aet_eta),
                                  C.POINTER(aet_delay), C.POINTER(i32), vp, vp]
    lib.aet_run_ticks.restype = C.c_int
    lib.aet_run_ticks.argtypes = [vp, C.POINTER(aet_threshold), C.POINTER(aet_eta),
                                  C.POINTER(aet_delay), C.c_float, i32, C.POINTER(i32)]
    lib.aet_server_aggregate.restype = C.c_int
    lib.aet_server_aggregate.argtypes = [vp, C.c_float, C.POINTER(i32), vp, vp]
    lib.aet_get_U.restype = C.c_int
    lib.aet_get_U.argtypes = [vp, i32, i32, vp, i32]
    lib.aet_get_weights.restype = C.c_int
    lib.aet_get_weights.argtypes = [vp, i32, vp, i32]
    lib.aet_get_round_info.restype = C.c_int
    lib.aet_get_round_info.argtypes = [vp, i32, i32, vp, vp]
    lib.aet_debug_sample_indices.restype = C.c_int
    lib.aet_debug_sample_indices.argtypes = [vp, i32, i64, i32, vp]
    lib.aet_all_done.restype = i32
    lib.aet_all_done.argtypes = [vp, i32]
    for name in ("aet_tick", "aet_inflight"):
        getattr(lib, name).restype = i64
        getattr(lib, name).argtypes = [vp]
    lib.aet_history.restype = i64
    lib.aet_history.argtypes = [vp, i32]
    lib.aet_synchronize.restype = C.c_int
    lib.aet_synchronize.argtypes = [vp]
    lib.aet_last_error.restype = C.c_char_p
    lib.aet_last_error.argtypes = [vp]
    lib.aet_reset.restype = C.c_int
    lib.aet_reset.argtypes = [vp]
    lib.aet_set_weights.restype = C.c_int
    lib.aet_set_weights.argtypes = [vp, i32, vp, i32]
    lib.aet_set_setup.restype = C.c_int
    lib.aet_set_setup.argtypes = [vp, vp, C.c_uint64]
    lib.aet_topology_workspace_bytes.restype = C.c_size_t
    lib.aet_topology_workspace_bytes.argtypes = [i32, i32]
    lib.aet_set_topology.restype = C.c_int
    lib.aet_set_topology.argtypes = [vp, vp, vp, vp, C.c_size_t]
    lib.aet_receive.restype = C.c_int
    lib.aet_receive.argtypes = [vp, C.c_float, C.POINTER(i32), vp, vp]
    lib.aet_profile_families.restype = i32
    lib.aet_profile_families.argtypes = []
    lib.aet_profile_family_name.restype = C.c_char_p
    lib.aet_profile_family_name.argtypes = [i32]
    lib.aet_profile_enable.restype = C.c_int
    lib.aet_profile_enable.argtypes = [vp, i32, i32]
    lib.aet_profile_read.restype = C.c_int
    lib.aet_profile_read.argtypes = [vp, i32, C.POINTER(i64), C.POINTER(C.c_double), i32]
    lib.aet_test_select_kernels.restype = None
    lib.aet_test_select_kernels.argtypes = [i32, i32]
    lib.aet_destroy.restype = None
    lib.aet_destroy.argtypes = [vp]
    _LIB = lib
    return lib


def model_desc(model) -> aet_model_desc:
    """Marshal a model description (in_c, in_h, in_w, layers[type,cout,k,pad,relu], batch)."""
    m = aet_model_desc()
    m.in_c, m.in_h, m.in_w = model.in_c, model.in_h, model.in_w
    m.n_layers, m.batch = len(model.layers), model.batch
    for j, L in enumerate(model.layers):
        m.layers[j] = aet_layer(L.type, L.cout, L.k, L.pad, L.relu)
    return m


def _hptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class AetSgd:
    """One library context.  Method names follow the C entry points."""

    def __init__(self, model, shards_X: Sequence[torch.Tensor], shards_y: Sequence[torch.Tensor],
                 w0: np.ndarray, seed: int, max_inflight: int = 1, max_rounds: int = 64,
                 stream: Optional[torch.cuda.Stream] = None, static_workspace: bool = False):
        """static_workspace: create the context with aet_init_static (the library's own
        workspace, w0 handed over as a device tensor) instead of aet_init."""
        self.lib = load_library()
        self.n = len(shards_X)
        self._desc = model_desc(model)
        self.P = int(self.lib.aet_n_params(C.byref(self._desc)))
        if self.P < 0:
            raise AetError(AET_EINVAL, "unsupported model description")
        for x, y in zip(shards_X, shards_y):
            if not (x.is_cuda and y.is_cuda and x.dtype == torch.float32 and y.dtype == torch.int32
                    and x.is_contiguous() and y.is_contiguous()):
                raise ValueError("shards must be contiguous CUDA tensors: float32 X, int32 y")
        self._keep = (list(shards_X), list(shards_y))
        self.device = shards_X[0].device
        nbytes = int(self.lib.aet_workspace_bytes(C.byref(self._desc), self.n, max_inflight, max_rounds))
        if nbytes == 0:
            raise AetError(AET_EINVAL, "aet_workspace_bytes rejected the arguments")
        self.workspace_bytes = nbytes
        if not static_workspace:
            self._ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
            base = self._ws.data_ptr()
            self._ws_ptr = (base + 255) & ~255
        sh = (aet_shard * self.n)()
        for c, (x, y) in enumerate(zip(shards_X, shards_y)):
            sh[c] = aet_shard(x.data_ptr(), y.data_ptr(), x.shape[0])
        self._w0 = np.ascontiguousarray(w0, dtype=np.float32)
        if self._w0.size != self.P:
            raise ValueError(f"w0 has {self._w0.size} entries, model has {self.P} parameters")
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        ctx = C.c_void_p()
        if static_workspace:
            self._w0_dev = torch.from_numpy(self._w0).to(self.device)
            torch.cuda.synchronize(self.device)
            rc = self.lib.aet_init_static(C.byref(ctx), C.byref(self._desc), self.n, sh,
                                          C.c_void_p(self._w0_dev.data_ptr()), C.c_uint64(seed),
                                          max_inflight, max_rounds, C.c_void_p(self.stream.cuda_stream))
        else:
            rc = self.lib.aet_init(C.byref(ctx), C.byref(self._desc), self.n, sh, _hptr(self._w0),
                                   C.c_uint64(seed), C.c_void_p(self._ws_ptr), nbytes, max_inflight,
                                   max_rounds, C.c_void_p(self.stream.cuda_stream))
        if rc != AET_OK:
            raise AetError(rc, self.lib.aet_last_error(None).decode())
        self.ctx = ctx
        self._cap = self.n * max_inflight
        self._fc = np.zeros(self.n, dtype=np.int32)
        self._fr = np.zeros(self.n, dtype=np.int32)
        self._ac = np.zeros(self._cap, dtype=np.int32)
        self._ar = np.zeros(self._cap, dtype=np.int32)

    def _check(self, rc: int):
        if rc != AET_OK:
            raise AetError(rc, self.lib.aet_last_error(self.ctx).decode())

    def aet_run_round(self, a: int, b: int, rounds: int, eta0: float, beta: float, power: float,
                      compute_factor: Optional[np.ndarray] = None,
                      is_straggler: Optional[np.ndarray] = None, delay_min: int = 0,
                      delay_max: int = 0, delay_seed: int = 0, d_max: int = -1) -> List[Tuple[int, int]]:
        thr = aet_threshold(a, b, rounds)
        eta = aet_eta(eta0, beta, power)
        cf = None if compute_factor is None else np.ascontiguousarray(compute_factor, dtype=np.int32)
        st = None if is_straggler is None else np.ascontiguousarray(is_straggler, dtype=np.uint8)
        dl = aet_delay(None if cf is None else cf.ctypes.data, None if st is None else st.ctypes.data,
                       delay_min, delay_max, delay_seed, d_max)
        nf = C.c_int32(0)
        self._check(self.lib.aet_run_round(self.ctx, C.byref(thr), C.byref(eta), C.byref(dl),
                                           C.byref(nf), _hptr(self._fc), _hptr(self._fr)))
        return list(zip(self._fc[: nf.value].tolist(), self._fr[: nf.value].tolist()))

    def aet_run_ticks(self, a: int, b: int, rounds: int, eta0: float, beta: float, power: float,
                      agg_scale: float, compute_factor: Optional[np.ndarray] = None,
                      is_straggler: Optional[np.ndarray] = None, delay_min: int = 0,
                      delay_max: int = 0, delay_seed: int = 0, d_max: int = -1,
                      max_ticks: int = 1 << 30) -> int:
        thr = aet_threshold(a, b, rounds)
        eta = aet_eta(eta0, beta, power)
        cf = None if compute_factor is None else np.ascontiguousarray(compute_factor, dtype=np.int32)
        st = None if is_straggler is None else np.ascontiguousarray(is_straggler, dtype=np.uint8)
        dl = aet_delay(None if cf is None else cf.ctypes.data, None if st is None else st.ctypes.data,
                       delay_min, delay_max, delay_seed, d_max)
        done = C.c_int32(0)
        self._check(self.lib.aet_run_ticks(self.ctx, C.byref(thr), C.byref(eta), C.byref(dl),
                                           C.c_float(agg_scale), max_ticks, C.byref(done)))
        return done.value

    def aet_server_aggregate(self, agg_scale: float) -> List[Tuple[int, int]]:
        na = C.c_int32(0)
        self._check(self.lib.aet_server_aggregate(self.ctx, C.c_float(agg_scale), C.byref(na),
                                                  _hptr(self._ac), _hptr(self._ar)))
        return list(zip(self._ac[: na.value].tolist(), self._ar[: na.value].tolist()))

    def aet_set_setup(self, weights: np.ndarray, seed: int):
        """Round lengths from the coin flips of Algorithm 1; p_c = weights[c] / sum."""
        w = np.ascontiguousarray(weights, dtype=np.uint32)
        if w.shape[0] != self.n:
            raise ValueError("weights needs n_clients entries")
        self._check(self.lib.aet_set_setup(self.ctx, _hptr(w), C.c_uint64(seed)))

    def aet_set_topology(self, nbr_off: np.ndarray, nbr: np.ndarray):
        """Peer-to-peer form on the given neighbour lists (CSR, host arrays)."""
        off = np.ascontiguousarray(nbr_off, dtype=np.int32)
        nb = np.ascontiguousarray(nbr, dtype=np.int32)
        if off.shape[0] != self.n + 1:
            raise ValueError("nbr_off needs n_clients + 1 entries")
        nbytes = int(self.lib.aet_topology_workspace_bytes(self.n, int(off[-1])))
        self._topo_ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        ptr = (self._topo_ws.data_ptr() + 255) & ~255
        self._check(self.lib.aet_set_topology(self.ctx, _hptr(off), _hptr(nb) if nb.size else None,
                                              C.c_void_p(ptr), nbytes))

    def aet_receive(self, scale: float) -> List[Tuple[int, int]]:
        na = C.c_int32(0)
        self._check(self.lib.aet_receive(self.ctx, C.c_float(scale), C.byref(na),
                                         _hptr(self._ac), _hptr(self._ar)))
        return list(zip(self._ac[: na.value].tolist(), self._ar[: na.value].tolist()))

    def aet_get_U(self, client: int, round_: int) -> np.ndarray:
        out = np.empty(self.P, dtype=np.float32)
        self._check(self.lib.aet_get_U(self.ctx, client, round_, _hptr(out), 1))
        return out

    def aet_get_weights(self, client: int = -1) -> np.ndarray:
        out = np.empty(self.P, dtype=np.float32)
        self._check(self.lib.aet_get_weights(self.ctx, client, _hptr(out), 1))
        return out

    def aet_set_weights(self, client: int, w: np.ndarray):
        w = np.ascontiguousarray(w, dtype=np.float32)
        if w.size != self.P:
            raise ValueError(f"got {w.size} values, the model has {self.P} parameters")
        self._check(self.lib.aet_set_weights(self.ctx, client, _hptr(w), 1))

    def aet_get_weights_device(self, client: int = -1) -> torch.Tensor:
        out = torch.empty(self.P, dtype=torch.float32, device=self.device)
        self._check(self.lib.aet_get_weights(self.ctx, client, C.c_void_p(out.data_ptr()), 0))
        return out

    def aet_get_round_info(self, client: int, round_: int) -> dict:
        ints = np.zeros(6, dtype=np.int64)
        dbl = np.zeros(2, dtype=np.float64)
        self._check(self.lib.aet_get_round_info(self.ctx, client, round_, _hptr(ints), _hptr(dbl)))
        return dict(s=int(ints[0]), m=int(ints[1]), q0=int(ints[2]), t0=int(ints[3]),
                    start_tick=int(ints[4]), arrival=int(ints[5]), eta=float(dbl[0]),
                    loss=float(dbl[1]))

    def aet_debug_sample_indices(self, client: int, q0: int, count: int) -> np.ndarray:
        out = np.empty(count, dtype=np.int32)
        self._check(self.lib.aet_debug_sample_indices(self.ctx, client, q0, count, _hptr(out)))
        return out

    def aet_all_done(self, rounds: int) -> bool:
        return bool(self.lib.aet_all_done(self.ctx, rounds))

    def aet_tick(self) -> int:
        return int(self.lib.aet_tick(self.ctx))

    def aet_history(self, client: int) -> int:
        return int(self.lib.aet_history(self.ctx, client))

    def aet_inflight(self) -> int:
        return int(self.lib.aet_inflight(self.ctx))

    def aet_synchronize(self):
        self._check(self.lib.aet_synchronize(self.ctx))

    def aet_reset(self):
        self._check(self.lib.aet_reset(self.ctx))

    def aet_profile_enable(self, family: int, on: bool):
        self._check(self.lib.aet_profile_enable(self.ctx, family, 1 if on else 0))

    def aet_profile_read(self, family: int, reset: bool = True) -> Tuple[int, float]:
        n, ms = C.c_int64(0), C.c_double(0.0)
        self._check(self.lib.aet_profile_read(self.ctx, family, C.byref(n), C.byref(ms),
                                              1 if reset else 0))
        return n.value, ms.value

    def profile_family_names(self) -> List[str]:
        return [self.lib.aet_profile_family_name(f).decode()
                for f in range(self.lib.aet_profile_families())]

    def aet_destroy(self):
        if getattr(self, "ctx", None):
            self.lib.aet_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.aet_destroy()
        except Exception:
            pass
