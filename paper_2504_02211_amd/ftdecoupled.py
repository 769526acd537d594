"""Thin ctypes binding of the decoupled fault-tolerant attention (include/ftdecoupled.h): argument
marshalling only; every step runs in the HIP library.  Raises if the library has not been built."""
from __future__ import annotations

import ctypes as C
from typing import Optional

import numpy as np

from .ftattn import device_pointer, load_library as _load

F16, BF16 = 0, 1
FT_OFF, FT_CORRECT = 0, 1
ST_GEMM1, ST_EXP, ST_PNORM, ST_GEMM2 = 0, 1, 2, 3
OK, EINVAL, EUNSUPPORTED, EHIP, ENOMEM = 0, -1, -2, -3, -4

EXPORTS = ("ftdec_create", "ftdec_get_config", "ftdec_footprint", "ftdec_forward", "ftdec_report", "ftdec_set_timing",
           "ftdec_get_timing", "ftdec_destroy", "ftdec_last_error")


class Config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("batch", C.c_int32), ("heads", C.c_int32), ("seq", C.c_int32),
                ("head_dim", C.c_int32), ("in_dtype", C.c_int32), ("causal", C.c_int32), ("softmax_scale", C.c_float),
                ("ft_mode", C.c_int32), ("tau_rel", C.c_float), ("eps_dmr", C.c_float), ("max_events", C.c_int32),
                ("device", C.c_int32)]


class Fault(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("b", "h", "stage", "row", "col", "bit")]


class Event(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("b", "h", "stage", "row", "col", "action")]


class ReportView(C.Structure):
    _fields_ = [("n_events", C.c_int32), ("n_events_dropped", C.c_int32), ("events", C.POINTER(Event)),
                ("retried_rows", C.c_int64)]


EVENT_DTYPE = np.dtype([(n, "<i4") for n in ("b", "h", "stage", "row", "col", "action")])


class FtDecError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"ftdec error {code}: {msg}")
        self.code = code


_ready = False


def load_library() -> C.CDLL:
    global _ready
    lib = _load()
    if not _ready:
        lib.ftdec_create.argtypes = [C.POINTER(Config), C.POINTER(C.c_void_p)]
        lib.ftdec_get_config.argtypes = [C.c_void_p, C.POINTER(Config)]
        lib.ftdec_footprint.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        lib.ftdec_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(Fault), C.c_int32,
                                      C.c_void_p]
        lib.ftdec_report.argtypes = [C.c_void_p, C.POINTER(ReportView)]
        lib.ftdec_set_timing.argtypes = [C.c_void_p, C.c_int32]
        lib.ftdec_get_timing.argtypes = [C.c_void_p, C.POINTER(C.c_float)]
        lib.ftdec_destroy.argtypes = [C.c_void_p]
        lib.ftdec_last_error.argtypes = [C.c_void_p]
        lib.ftdec_last_error.restype = C.c_char_p
        for n in EXPORTS[:-1]:
            getattr(lib, n).restype = C.c_int
        _ready = True
    return lib


class Report:
    def __init__(self, view: ReportView):
        n = view.n_events
        self.n_events, self.n_events_dropped, self.retried_rows = n, view.n_events_dropped, int(view.retried_rows)
        self.events = (np.frombuffer(C.string_at(view.events, n * C.sizeof(Event)), dtype=EVENT_DTYPE).copy() if n
                       else np.zeros(0, dtype=EVENT_DTYPE))

    def event_set(self):
        """Set of (b, h, stage, row, col) tuples."""
        e = self.events
        return set(zip(e["b"].tolist(), e["h"].tolist(), e["stage"].tolist(), e["row"].tolist(), e["col"].tolist()))


class FtDecoupled:
    """One context of the decoupled scheme (one shape, one device)."""

    def __init__(self, batch: int, heads: int, seq: int, head_dim: int, in_dtype: int, causal: bool,
                 ft_mode: int = FT_CORRECT, softmax_scale: float = 0.0, tau_rel: float = 0.0, eps_dmr: float = 0.0,
                 max_events: int = 0, device: int = 0):
        self.lib = load_library()
        cfg = Config(C.sizeof(Config), batch, heads, seq, head_dim, in_dtype, int(bool(causal)), softmax_scale, ft_mode,
                     tau_rel, eps_dmr, max_events, device)
        self.handle = C.c_void_p()
        rc = self.lib.ftdec_create(C.byref(cfg), C.byref(self.handle))
        if rc != OK:
            self.handle = C.c_void_p()
            raise FtDecError(rc, self.lib.ftdec_last_error(None).decode())
        eff = Config()
        self.lib.ftdec_get_config(self.handle, C.byref(eff))
        self.config = eff

    def _check(self, rc: int) -> None:
        if rc != OK:
            raise FtDecError(rc, self.lib.ftdec_last_error(self.handle).decode())

    def footprint(self):
        """(total device bytes of the context, bytes of S and P)."""
        a, b = C.c_int64(), C.c_int64()
        self._check(self.lib.ftdec_footprint(self.handle, C.byref(a), C.byref(b)))
        return int(a.value), int(b.value)

    def forward(self, q, k, v, o, faults: Optional[np.ndarray] = None, stream: int = 0) -> None:
        """q, k, v: device tensors of the input type, o: fp32; faults: int32 [n, 6] of (b, h, stage, row, col, bit)."""
        c = self.config
        ne = c.batch * c.heads * c.seq * c.head_dim
        n, fp = 0, None
        if faults is not None and len(faults):
            fa = np.ascontiguousarray(faults, dtype=np.int32).reshape(-1, 6)
            n, fp = fa.shape[0], fa.ctypes.data_as(C.POINTER(Fault))
        self._check(self.lib.ftdec_forward(self.handle, device_pointer(q, "q", ne, c.in_dtype, c.device),
                                           device_pointer(k, "k", ne, c.in_dtype, c.device),
                                           device_pointer(v, "v", ne, c.in_dtype, c.device),
                                           device_pointer(o, "o", ne, 2, c.device), fp, n, C.c_void_p(stream)))

    def report(self) -> Report:
        view = ReportView()
        self._check(self.lib.ftdec_report(self.handle, C.byref(view)))
        return Report(view)

    def set_timing(self, enabled: bool) -> None:
        self._check(self.lib.ftdec_set_timing(self.handle, int(enabled)))

    def get_timing(self):
        """(ABFT-GEMM I ms, DMR softmax ms, ABFT-GEMM II ms) of the last forward; needs set_timing(True)."""
        ms = (C.c_float * 3)()
        self._check(self.lib.ftdec_get_timing(self.handle, ms))
        return float(ms[0]), float(ms[1]), float(ms[2])

    def close(self) -> None:
        if self.handle:
            self.lib.ftdec_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
