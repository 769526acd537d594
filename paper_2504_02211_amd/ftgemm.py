"""Thin ctypes binding of the fault-tolerant linear layer in libftattn.so: argument marshalling only.

The contraction, the checksum encoding, verification and repair all run inside the HIP library;
this module passes device pointers of torch tensors and copies the host-side report into numpy
arrays.  It raises if the library has not been built -- there is no fallback.
"""
from __future__ import annotations

import ctypes as C
from typing import Optional

import numpy as np

from . import ftattn as _base

F16, BF16, F32 = 0, 1, 2
FT_OFF, FT_CORRECT, FT_DETECT = 0, 1, 2
OK, EINVAL, EUNSUPPORTED, EHIP, ENOMEM, ESTATE = 0, -1, -2, -3, -4, -5

EXPORTS = ("ftgemm_create", "ftgemm_get_config", "ftgemm_encode_weights", "ftgemm_forward", "ftgemm_report",
           "ftgemm_set_timing", "ftgemm_get_timing", "ftgemm_destroy", "ftgemm_last_error")


class Config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("m", C.c_int32), ("n", C.c_int32), ("k", C.c_int32),
                ("in_dtype", C.c_int32), ("out_dtype", C.c_int32), ("ft_mode", C.c_int32), ("stride", C.c_int32),
                ("block_n", C.c_int32), ("tau_rel", C.c_float), ("tau_abs", C.c_float), ("fold_tokens", C.c_int32),
                ("max_events", C.c_int32), ("device", C.c_int32)]


class Fault(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("row", "col", "bit")]


class Event(C.Structure):
    _fields_ = [("row", C.c_int32), ("col", C.c_int32), ("residual", C.c_float), ("action", C.c_int32)]


class ReportView(C.Structure):
    _fields_ = [("n_events", C.c_int32), ("n_events_dropped", C.c_int32), ("events", C.POINTER(Event)),
                ("residual_max", C.c_float)]


EVENT_DTYPE = np.dtype([("row", "<i4"), ("col", "<i4"), ("residual", "<f4"), ("action", "<i4")])

_typed = False


class FtGemmError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"ftgemm error {code}: {msg}")
        self.code = code


def load_library() -> C.CDLL:
    """The shared library with the ftgemm_* prototypes set; raises if it is not built."""
    global _typed
    lib = _base.load_library()
    if not _typed:
        lib.ftgemm_create.argtypes = [C.POINTER(Config), C.POINTER(C.c_void_p)]
        lib.ftgemm_get_config.argtypes = [C.c_void_p, C.POINTER(Config)]
        lib.ftgemm_encode_weights.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        lib.ftgemm_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(Fault), C.c_int32,
                                       C.c_void_p]
        lib.ftgemm_report.argtypes = [C.c_void_p, C.POINTER(ReportView)]
        lib.ftgemm_set_timing.argtypes = [C.c_void_p, C.c_int32]
        lib.ftgemm_get_timing.argtypes = [C.c_void_p, C.POINTER(C.c_float)]
        lib.ftgemm_destroy.argtypes = [C.c_void_p]
        lib.ftgemm_last_error.argtypes = [C.c_void_p]
        lib.ftgemm_last_error.restype = C.c_char_p
        for n in EXPORTS:
            if n != "ftgemm_last_error":
                getattr(lib, n).restype = C.c_int
        _typed = True
    return lib


class Report:
    """Host copy of ftgemm_report's view."""

    def __init__(self, view: ReportView):
        n = view.n_events
        self.n_events = n
        self.n_events_dropped = view.n_events_dropped
        self.residual_max = float(view.residual_max)
        if n:
            self.events = np.frombuffer(C.string_at(view.events, n * C.sizeof(Event)), dtype=EVENT_DTYPE).copy()
        else:
            self.events = np.zeros(0, dtype=EVENT_DTYPE)

    def event_list(self):
        """Sorted list of (row, col, action)."""
        e = self.events
        return sorted(zip(e["row"].tolist(), e["col"].tolist(), e["action"].tolist()))


class FtGemm:
    """One context of the C library: Y = X W^T for one (m, n, k) on one device."""

    def __init__(self, m: int, n: int, k: int, out_dtype: int = F32, ft_mode: int = FT_CORRECT, tau_rel: float = 0.0,
                 tau_abs: float = -1.0, max_events: int = 0, device: int = 0, in_dtype: int = F16,
                 fold_tokens: bool = False):
        self.lib = load_library()
        cfg = Config(C.sizeof(Config), m, n, k, in_dtype, out_dtype, ft_mode, 8, 0, tau_rel, tau_abs, int(bool(fold_tokens)),
                     max_events, device)
        self.handle = C.c_void_p()
        rc = self.lib.ftgemm_create(C.byref(cfg), C.byref(self.handle))
        if rc != OK:
            self.handle = C.c_void_p()
            raise FtGemmError(rc, self.lib.ftgemm_last_error(None).decode())
        eff = Config()
        self.lib.ftgemm_get_config(self.handle, C.byref(eff))
        self.config = eff

    def _check(self, rc: int) -> None:
        if rc != OK:
            raise FtGemmError(rc, self.lib.ftgemm_last_error(self.handle).decode())

    def _ptr(self, t, name: str) -> C.c_void_p:
        """Device address of x / w / y, checked against the context's shape (see ftattn.device_pointer)."""
        from .ftattn import device_pointer
        c = self.config
        n_elems, dt = {"x": (c.m * c.k, c.in_dtype), "w": (c.n * c.k, c.in_dtype), "y": (c.m * c.n, c.out_dtype)}[name]
        return device_pointer(t, name, n_elems, dt, c.device)

    def encode_weights(self, w, stream: int = 0) -> None:
        self._check(self.lib.ftgemm_encode_weights(self.handle, self._ptr(w, "w"), C.c_void_p(stream)))

    def forward(self, x, w, y, faults: Optional[np.ndarray] = None, stream: int = 0) -> None:
        """x, w, y: objects with data_ptr() (torch device tensors) or integer device addresses.
        faults: int32 array [n, 3] of (row, col, bit)."""
        n = 0
        fp = None
        if faults is not None and len(faults):
            fa = np.ascontiguousarray(faults, dtype=np.int32).reshape(-1, 3)
            n = fa.shape[0]
            fp = fa.ctypes.data_as(C.POINTER(Fault))
        self._check(self.lib.ftgemm_forward(self.handle, self._ptr(x, "x"), self._ptr(w, "w"), self._ptr(y, "y"), fp, n,
                                            C.c_void_p(stream)))

    def report(self) -> Report:
        view = ReportView()
        self._check(self.lib.ftgemm_report(self.handle, C.byref(view)))
        return Report(view)

    def set_timing(self, enabled: bool) -> None:
        self._check(self.lib.ftgemm_set_timing(self.handle, int(enabled)))

    def get_timing(self) -> float:
        """Kernel milliseconds of the last forward; needs set_timing(True)."""
        ms = C.c_float()
        self._check(self.lib.ftgemm_get_timing(self.handle, C.byref(ms)))
        return float(ms.value)

    def close(self) -> None:
        if self.handle:
            self.lib.ftgemm_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
