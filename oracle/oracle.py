"""ctypes front end of the CPU oracle (oracle/adseq_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's CPU-baseline leg.  The product package never imports this module.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adseq_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

RING, FIFO, SORTED, SYN_FIFO, SYN_LATEST, SYN_BINS = 0, 1, 2, 3, 4, 5
SURR_SUPERSPIKE, SURR_OFF, GRAD_SPIKE_TIME = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler (no GPU code)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared",
                               "-pthread", "-o", _LIB, _SRC])
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [
        ("n_neurons", C.c_int32), ("batch", C.c_int32), ("d_max_steps", C.c_int32),
        ("capacity", C.c_int32), ("kind", C.c_int32), ("n_steps", C.c_int32),
        ("surrogate", C.c_int32), ("exact_f64", C.c_int32),
        ("dt_ms", C.c_float), ("tau_m_ms", C.c_float), ("v_thresh", C.c_float),
        ("v_reset", C.c_float), ("ext_rate_hz", C.c_float), ("ext_weight", C.c_float),
        ("seed", C.c_uint64), ("n_synapses", C.c_int64),
        ("row_ptr", C.c_void_p), ("col", C.c_void_p), ("weight", C.c_void_p),
        ("delay_steps", C.c_void_p), ("delay_ms", C.c_void_p),
        ("i_ext", C.c_void_p), ("forced_spikes", C.c_void_p),
        ("log_events", C.c_int32), ("keep_currents", C.c_int32), ("n_threads", C.c_int32),
        ("tau_syn_ms", C.c_float), ("tau_rise_ms", C.c_float),
        ("progress_file", C.c_char_p),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.oracle_forward.restype = C.c_void_p
        L.oracle_forward.argtypes = [C.POINTER(_Cfg)]
        for name, rt in [("oracle_U", C.POINTER(C.c_float)), ("oracle_U64", C.POINTER(C.c_double)),
                         ("oracle_S", C.POINTER(C.c_uint8)), ("oracle_I", C.POINTER(C.c_float)),
                         ("oracle_Iq", C.POINTER(C.c_int32)), ("oracle_D", C.POINTER(C.c_int32)),
                         ("oracle_aq", C.POINTER(C.c_int32)), ("oracle_af", C.POINTER(C.c_float)),
                         ("oracle_ff", C.POINTER(C.c_float)), ("oracle_ad", C.POINTER(C.c_double))]:
            getattr(L, name).restype = rt
            getattr(L, name).argtypes = [C.c_void_p]
        L.oracle_status.restype = C.c_int
        L.oracle_status.argtypes = [C.c_void_p]
        L.oracle_counters.argtypes = [C.c_void_p, C.POINTER(C.c_int64)]
        L.oracle_event_log.restype = C.c_int64
        L.oracle_event_log.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.POINTER(C.c_int64)),
                                       C.POINTER(C.POINTER(C.c_int32)), C.POINTER(C.POINTER(C.c_int32)),
                                       C.POINTER(C.POINTER(C.c_int32))]
        L.oracle_backward.restype = C.c_int
        L.oracle_backward.argtypes = [C.c_void_p] + [C.c_void_p] * 5
        L.oracle_free.argtypes = [C.c_void_p]
        L.oracle_exp_neg.restype = C.c_double
        L.oracle_exp_neg.argtypes = [C.c_double]
        L.oracle_drive_bits.restype = C.c_uint32
        L.oracle_drive_bits.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64]
        L.oracle_mix64.restype = C.c_uint64
        L.oracle_mix64.argtypes = [C.c_uint64]
        _lib = L
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


class OracleError(RuntimeError):
    pass


class Run:
    """One forward simulation; holds the tape so that backward() can follow."""

    def __init__(self, wl, kind: int = RING, capacity: int = 0, *, n_steps: Optional[int] = None,
                 batch: Optional[int] = None, surrogate: int = 0, exact_f64: bool = False,
                 i_ext: Optional[np.ndarray] = None, forced_spikes: Optional[np.ndarray] = None,
                 log_events: bool = False, keep_currents: bool = False, n_threads: int = 1):
        L = lib()
        self.wl = wl
        self.T = wl.n_steps if n_steps is None else n_steps
        self.B = wl.batch if batch is None else batch
        self.N = wl.n_neurons
        self.S = wl.n_synapses
        # keep references so the arrays outlive the C object
        self._keep = dict(
            row_ptr=np.ascontiguousarray(wl.row_ptr, dtype=np.int64),
            col=np.ascontiguousarray(wl.col, dtype=np.int32),
            weight=np.ascontiguousarray(wl.weight, dtype=np.float32),
            delay_steps=None if wl.delay_steps is None else np.ascontiguousarray(wl.delay_steps, dtype=np.uint8),
            delay_ms=None if wl.delay_ms is None else np.ascontiguousarray(wl.delay_ms, dtype=np.float32),
            i_ext=None if i_ext is None else np.ascontiguousarray(i_ext, dtype=np.float32),
            forced=None if forced_spikes is None else np.ascontiguousarray(forced_spikes, dtype=np.uint8),
        )
        k = self._keep
        shape = (self.T, self.B, self.N)
        for name in ("i_ext", "forced"):
            if k[name] is not None and k[name].shape != shape:
                raise ValueError(f"{name} must have shape {shape}")
        cfg = _Cfg(n_neurons=self.N, batch=self.B, d_max_steps=wl.d_max_steps, capacity=capacity,
                   kind=kind, n_steps=self.T, surrogate=surrogate, exact_f64=int(exact_f64),
                   dt_ms=wl.dt_ms, tau_m_ms=wl.tau_m_ms, v_thresh=wl.v_thresh, v_reset=wl.v_reset,
                   ext_rate_hz=wl.ext_rate_hz, ext_weight=wl.ext_weight, seed=wl.seed,
                   n_synapses=self.S, row_ptr=_ptr(k["row_ptr"]), col=_ptr(k["col"]),
                   weight=_ptr(k["weight"]), delay_steps=_ptr(k["delay_steps"]),
                   delay_ms=_ptr(k["delay_ms"]), i_ext=_ptr(k["i_ext"]),
                   forced_spikes=_ptr(k["forced"]), log_events=int(log_events),
                   keep_currents=int(keep_currents), n_threads=n_threads,
                   tau_syn_ms=float(getattr(wl, "tau_syn_ms", 0.0)),
                   tau_rise_ms=float(getattr(wl, "tau_rise_ms", 0.0)),
                   # (read from Python's own copy of the environment: the C side never calls getenv)
                   progress_file=(os.environ.get("ORACLE_PROGRESS_FILE") or "").encode() or None)
        self._exact = bool(exact_f64)
        self._keep_currents = keep_currents
        self._h = L.oracle_forward(C.byref(cfg))
        st = L.oracle_status(self._h)
        if st != 0:
            L.oracle_free(self._h)
            self._h = None
            raise OracleError({-1: "invalid argument", -2: "delay out of range"}.get(st, str(st)))

    def _arr(self, fn, dtype, shape):
        p = getattr(lib(), fn)(self._h)
        n = int(np.prod(shape))
        if n == 0:
            return np.zeros(shape, dtype=dtype)
        return np.ctypeslib.as_array(p, shape=(n,)).view(dtype).reshape(shape).copy()

    @property
    def U(self):
        return self._arr("oracle_U", np.float32, (self.T, self.B, self.N))

    @property
    def U64(self):
        assert self._exact
        return self._arr("oracle_U64", np.float64, (self.T, self.B, self.N))

    @property
    def spikes(self):
        return self._arr("oracle_S", np.uint8, (self.T, self.B, self.N))

    @property
    def I(self):
        return self._arr("oracle_I", np.float32, (self.T, self.B, self.N))

    @property
    def Iq(self):
        assert self._keep_currents
        return self._arr("oracle_Iq", np.int32, (self.T, self.B, self.N))

    @property
    def D(self):
        return self._arr("oracle_D", np.int32, (self.S,))

    @property
    def a_q(self):
        return self._arr("oracle_aq", np.int32, (self.S,))

    @property
    def a_f(self):
        return self._arr("oracle_af", np.float32, (self.S,))

    @property
    def f_f(self):
        return self._arr("oracle_ff", np.float32, (self.S,))

    @property
    def a_d(self):
        return self._arr("oracle_ad", np.float64, (self.S,))

    def counters(self):
        out = (C.c_int64 * 9)()
        lib().oracle_counters(self._h, out)
        names = ["enqueued", "dropped", "delivered", "in_flight", "sum_enqueued", "sum_dropped",
                 "sum_delivered", "sum_in_flight", "max_occupancy"]
        return dict(zip(names, [int(x) for x in out]))

    def event_log(self, which: str):
        """'delivered' or 'dropped' -> dict of arrays syn, n_emit, k, b (log order)."""
        syn = C.POINTER(C.c_int64)()
        ne = C.POINTER(C.c_int32)()
        kk = C.POINTER(C.c_int32)()
        bb = C.POINTER(C.c_int32)()
        n = lib().oracle_event_log(self._h, 0 if which == "delivered" else 1, C.byref(syn),
                                   C.byref(ne), C.byref(kk), C.byref(bb))
        if n == 0:
            z32 = np.zeros(0, np.int32)
            return dict(syn=np.zeros(0, np.int64), n_emit=z32, k=z32.copy(), b=z32.copy())
        f = lambda p: np.ctypeslib.as_array(p, shape=(n,)).copy()
        return dict(syn=f(syn), n_emit=f(ne), k=f(kk), b=f(bb))

    def backward(self, dL_dcount: Optional[np.ndarray] = None, dL_dU: Optional[np.ndarray] = None,
                 want_gU: bool = False):
        """Reverse-mode gradients in fp64: (grad_w [S], grad_d [S]) (+ dL/dU [T,B,N])."""
        dc = None if dL_dcount is None else np.ascontiguousarray(dL_dcount, dtype=np.float32)
        du = None if dL_dU is None else np.ascontiguousarray(dL_dU, dtype=np.float32)
        if dc is not None:
            assert dc.shape == (self.B, self.N)
        if du is not None:
            assert du.shape == (self.T, self.B, self.N)
        gw = np.zeros(self.S, np.float64)
        gd = np.zeros(self.S, np.float64)
        gU = np.zeros((self.T, self.B, self.N), np.float64) if want_gU else None
        st = lib().oracle_backward(self._h, _ptr(dc), _ptr(du), _ptr(gw), _ptr(gd), _ptr(gU))
        if st != 0:
            raise OracleError(str(st))
        return (gw, gd, gU) if want_gU else (gw, gd)

    def close(self):
        if getattr(self, "_h", None):
            lib().oracle_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def mix64(z: int) -> int:
    return int(lib().oracle_mix64(C.c_uint64(z)))


def drive_bits(seed: int, g: int, n: int) -> int:
    return int(lib().oracle_drive_bits(C.c_uint64(seed), C.c_uint64(g), C.c_uint64(n)))


def exp_neg(x: float) -> float:
    return float(lib().oracle_exp_neg(C.c_double(x)))
