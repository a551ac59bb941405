"""Thin ctypes binding over libadseq.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in
include/adseq.h; PyTorch is used for device memory and the current stream.
There is no CPU fallback: loading fails loudly if the library is not built.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ADSEQ_LIB", os.path.join(_HERE, "libadseq.so"))

RING, FIFO, SORTED, SYN_FIFO, SYN_LATEST, SYN_BINS = 0, 1, 2, 3, 4, 5
SURR_SUPERSPIKE, SURR_OFF, GRAD_SPIKE_TIME = 0, 1, 2

ERRORS = {0: "OK", -1: "INVALID_ARG", -2: "DELAY_RANGE", -3: "WORKSPACE", -4: "ORDER",
          -5: "NO_TAPE", -6: "HIP", -7: "CAPACITY", -8: "GRAPH", -9: "HOST_MEMORY"}
STATIC_WORKSPACE_BYTES = 32 << 20

EXPORTS = ["adseq_workspace_bytes", "adseq_create", "adseq_create_static", "adseq_destroy", "adseq_reset", "adseq_deliver",
           "adseq_enqueue", "adseq_run_open", "adseq_step", "adseq_run", "adseq_backward", "adseq_drop_count",
           "adseq_counters", "adseq_tape", "adseq_spike_counts", "adseq_profile", "adseq_profile_read", "adseq_last_error"]


class AdseqError(RuntimeError):
    def __init__(self, code: int, text: str = ""):
        self.code = code
        super().__init__(f"adseq error {code} ({ERRORS.get(code, '?')}) {text}")


class Config(C.Structure):
    _fields_ = [
        ("n_neurons", C.c_int32), ("batch", C.c_int32), ("d_max_steps", C.c_int32),
        ("capacity", C.c_int32), ("kind", C.c_int32), ("surrogate", C.c_int32),
        ("record_tape", C.c_int32), ("max_steps", C.c_int32),
        ("dt_ms", C.c_float), ("tau_m_ms", C.c_float), ("v_thresh", C.c_float), ("v_reset", C.c_float),
        ("ext_rate_hz", C.c_float), ("ext_weight", C.c_float),
        ("tau_syn_ms", C.c_float), ("tau_rise_ms", C.c_float),
        ("seed", C.c_uint64), ("n_synapses", C.c_int64),
        ("row_ptr", C.c_void_p), ("col", C.c_void_p), ("weight", C.c_void_p),
        ("delay_steps", C.c_void_p), ("delay_ms", C.c_void_p),
        ("tape_spike_capacity", C.c_int64), ("tape_event_capacity", C.c_int64),
        ("step_event_capacity", C.c_int64),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("stream", C.c_void_p),
    ]


class TapeView(C.Structure):
    _fields_ = [("membrane", C.c_void_p), ("step_offset", C.c_void_p), ("spike_id", C.c_void_p),
                ("event_base", C.c_void_p), ("admitted", C.c_void_p), ("steps_recorded", C.c_int64)]


_lib = None


def load():
    """Loads the in-tree HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                               "(python -m paper_2512_05906_amd.build); there is no fallback path")
        L = C.CDLL(LIB_PATH)
        vp, i64 = C.c_void_p, C.c_int64
        L.adseq_workspace_bytes.restype = C.c_size_t
        L.adseq_workspace_bytes.argtypes = [C.POINTER(Config)]
        L.adseq_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
        L.adseq_create_static.argtypes = [C.POINTER(Config), C.POINTER(vp)]
        L.adseq_destroy.argtypes = [vp]
        L.adseq_reset.argtypes = [vp, vp]
        L.adseq_deliver.argtypes = [vp, i64, vp, vp]
        L.adseq_enqueue.argtypes = [vp, i64, vp, vp, vp]
        L.adseq_step.argtypes = [vp, i64, vp, vp, vp]
        L.adseq_run_open.argtypes = [vp, i64, i64, vp, vp, vp, vp, i64, vp]
        L.adseq_run.argtypes = [vp, i64, i64, vp]
        L.adseq_backward.argtypes = [vp, vp, vp, vp, vp, vp]
        L.adseq_drop_count.argtypes = [vp, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64),
                                       C.POINTER(C.c_uint64), vp]
        L.adseq_counters.argtypes = [vp, C.POINTER(i64), vp]
        L.adseq_tape.argtypes = [vp, C.POINTER(TapeView)]
        L.adseq_spike_counts.argtypes = [vp, vp, vp]
        L.adseq_profile.argtypes = [vp, C.c_int]
        L.adseq_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64), vp]
        L.adseq_last_error.restype = C.c_char_p
        L.adseq_last_error.argtypes = [vp]
        for name in EXPORTS:
            if name not in ("adseq_workspace_bytes", "adseq_last_error"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


class _RawDeviceBytes:
    """nbytes of device memory at a raw address, for torch.as_tensor (zero-copy view)."""

    def __init__(self, ptr: int, nbytes: int):
        self.__cuda_array_interface__ = {"shape": (nbytes,), "typestr": "|u1", "data": (ptr, False), "version": 2}


def _copy_out(ptr: int, nbytes: int, dev) -> torch.Tensor:
    """uint8 view of device memory that no tensor owns (the library's static workspace)."""
    if nbytes == 0:
        return torch.empty(0, dtype=torch.uint8, device=dev)
    return torch.as_tensor(_RawDeviceBytes(ptr, nbytes), device=dev)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


class Adseq:
    """One network x `batch` trials on the current CUDA (HIP) device."""

    def __init__(self, wl, kind: int = RING, capacity: int = 0, *, batch: Optional[int] = None,
                 record_tape: bool = False, max_steps: Optional[int] = None,
                 surrogate: int = SURR_SUPERSPIKE, tape_spike_capacity: int = 0,
                 tape_event_capacity: int = 0, step_event_capacity: int = 0,
                 device: str = "cuda:0", static_workspace: bool = False):
        self.lib = load()
        self.dev = torch.device(device)
        self.N, self.B = wl.n_neurons, wl.batch if batch is None else batch
        self.S = wl.n_synapses
        self.kind = kind
        up = lambda a, dt: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=dt)).to(self.dev)
        # caller-owned CSR on the device (kept alive with the handle)
        self.row_ptr = up(wl.row_ptr, np.int64)
        self.col = up(wl.col, np.int32)
        self.weight = up(wl.weight, np.float32)
        self.delay_steps = up(wl.delay_steps, np.uint8)
        self.delay_ms = up(wl.delay_ms, np.float32)
        self.max_steps = (wl.n_steps if max_steps is None else max_steps) if record_tape else 0
        cfg = Config(n_neurons=self.N, batch=self.B, d_max_steps=wl.d_max_steps, capacity=capacity,
                     kind=kind, surrogate=surrogate, record_tape=int(record_tape),
                     max_steps=self.max_steps, dt_ms=wl.dt_ms, tau_m_ms=wl.tau_m_ms,
                     v_thresh=wl.v_thresh, v_reset=wl.v_reset, ext_rate_hz=wl.ext_rate_hz,
                     ext_weight=wl.ext_weight, tau_syn_ms=float(getattr(wl, "tau_syn_ms", 0.0)),
                     tau_rise_ms=float(getattr(wl, "tau_rise_ms", 0.0)), seed=wl.seed,
                     n_synapses=self.S,
                     row_ptr=_dptr(self.row_ptr), col=_dptr(self.col), weight=_dptr(self.weight),
                     delay_steps=_dptr(self.delay_steps), delay_ms=_dptr(self.delay_ms),
                     tape_spike_capacity=tape_spike_capacity, tape_event_capacity=tape_event_capacity,
                     step_event_capacity=step_event_capacity)
        nbytes = self.lib.adseq_workspace_bytes(C.byref(cfg))
        if nbytes == 0:
            raise AdseqError(-1, "adseq_workspace_bytes rejected the configuration")
        self.workspace = None
        if not static_workspace:
            self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.dev)
            base = self.workspace.data_ptr()
            cfg.workspace = (base + 255) & ~255
            cfg.workspace_bytes = nbytes
        with torch.cuda.device(self.dev):
            cfg.stream = _stream()
            h = C.c_void_p()
            if static_workspace:   # the library's own workspace: nothing is allocated
                rc = self.lib.adseq_create_static(C.byref(cfg), C.byref(h))
            else:
                rc = self.lib.adseq_create(C.byref(cfg), C.byref(h))
        if rc != 0:
            raise AdseqError(rc, "adseq_create_static" if static_workspace else "adseq_create")
        self.h = h
        self.cfg = cfg
        self.workspace_bytes = nbytes

    def _check(self, rc: int):
        if rc != 0:
            raise AdseqError(rc, self.lib.adseq_last_error(self.h).decode())

    def reset(self):
        self._check(self.lib.adseq_reset(self.h, _stream()))

    def step(self, n: int, i_ext: Optional[torch.Tensor] = None, spikes_out: Optional[torch.Tensor] = None):
        self._check(self.lib.adseq_step(self.h, n, _dptr(i_ext), _dptr(spikes_out), _stream()))

    def run(self, step0: int, n_steps: int):
        self._check(self.lib.adseq_run(self.h, step0, n_steps, _stream()))

    def deliver(self, n: int, I_out: torch.Tensor):
        self._check(self.lib.adseq_deliver(self.h, n, _dptr(I_out), _stream()))

    def enqueue(self, n: int, spike_ids: torch.Tensor, n_spikes: torch.Tensor):
        self._check(self.lib.adseq_enqueue(self.h, n, _dptr(spike_ids), _dptr(n_spikes), _stream()))

    def run_open(self, step0: int, n_steps: int, spike_ids: torch.Tensor, spike_offsets: np.ndarray,
                 n_spikes: torch.Tensor, I_out: torch.Tensor, I_stride: int):
        """n_steps x (deliver, enqueue); spike_offsets is a host int64 array [n_steps]."""
        offs = np.ascontiguousarray(spike_offsets, dtype=np.int64)
        self._check(self.lib.adseq_run_open(self.h, step0, n_steps, _dptr(spike_ids), offs.ctypes.data,
                                            _dptr(n_spikes), _dptr(I_out), I_stride, _stream()))

    def backward(self, dL_dcount: Optional[torch.Tensor], dL_dU: Optional[torch.Tensor],
                 grad_w: torch.Tensor, grad_d: torch.Tensor):
        self._check(self.lib.adseq_backward(self.h, _dptr(dL_dcount), _dptr(dL_dU), _dptr(grad_w),
                                            _dptr(grad_d), _stream()))

    def drop_count(self):
        d, e, v = C.c_uint64(), C.c_uint64(), C.c_uint64()
        self._check(self.lib.adseq_drop_count(self.h, C.byref(d), C.byref(e), C.byref(v), _stream()))
        return dict(dropped=d.value, enqueued=e.value, delivered=v.value)

    def counters(self):
        out = (C.c_int64 * 8)()
        self._check(self.lib.adseq_counters(self.h, out, _stream()))
        names = ["enqueued", "dropped", "delivered", "sum_enqueued", "sum_dropped", "sum_delivered",
                 "tape_spikes", "error_bits"]
        return dict(zip(names, [int(x) for x in out]))

    def spike_counts(self, counts: torch.Tensor):
        """Per-(trial, neuron) spike counts of the recorded run into an int32 tensor [B*N]."""
        self._check(self.lib.adseq_spike_counts(self.h, _dptr(counts), _stream()))

    def profile(self, enable: bool):
        self._check(self.lib.adseq_profile(self.h, int(enable)))

    def profile_read(self):
        ms = (C.c_double * 4)()
        cnt = (C.c_int64 * 4)()
        self._check(self.lib.adseq_profile_read(self.h, ms, cnt, _stream()))
        names = ["fan_out", "lif", "bwd_gather", "bwd_neurons"]
        return {k: dict(ms=ms[i], launches=int(cnt[i])) for i, k in enumerate(names)}

    def tape(self):
        """Zero-copy torch views of the tape inside the workspace."""
        tv = TapeView()
        self._check(self.lib.adseq_tape(self.h, C.byref(tv)))
        BN = self.B * self.N

        def view(ptr, nbytes, dtype):
            if self.workspace is None:   # the library's static workspace is no torch tensor: copy out
                return _copy_out(ptr, nbytes, self.dev).view(dtype)
            off = ptr - self.workspace.data_ptr()
            return self.workspace[off:off + nbytes].view(dtype)

        T = int(tv.steps_recorded)
        out = dict(steps=T)
        out["U"] = view(tv.membrane, T * BN * 4, torch.float32).view(T, self.B, self.N)
        if not tv.step_offset:      # ring: the spikes are U >= v_thresh, no list is kept
            return out
        off = view(tv.step_offset, (T + 1) * 8, torch.int64)
        out["step_offset"] = off
        n_spk = int(off[T].item()) if T > 0 else 0
        out["spike_id"] = view(tv.spike_id, n_spk * 4, torch.int32)
        if tv.event_base:
            out["event_base"] = view(tv.event_base, n_spk * 8, torch.int64)
            out["admitted_ptr"] = tv.admitted
            out["_view"] = view
        return out

    def membrane_tape(self, n_steps: int) -> torch.Tensor:
        """Zero-copy view [n_steps, B, N] of the recorded membrane values (no synchronisation)."""
        tv = TapeView()
        self._check(self.lib.adseq_tape(self.h, C.byref(tv)))
        off = tv.membrane - self.workspace.data_ptr()
        nb = n_steps * self.B * self.N * 4
        return self.workspace[off:off + nb].view(torch.float32).view(n_steps, self.B, self.N)

    def admitted_flags(self, event_base: int, count: int) -> torch.Tensor:
        tv = TapeView()
        self._check(self.lib.adseq_tape(self.h, C.byref(tv)))
        off = tv.admitted - self.workspace.data_ptr() + event_base
        return self.workspace[off:off + count]

    def close(self):
        if getattr(self, "h", None):
            self.lib.adseq_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
