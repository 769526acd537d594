"""Thin ctypes binding of libftattn.so: argument marshalling only.

Every step of the attention pass runs inside the HIP library; this module passes
device pointers of torch tensors and copies the host-side report into numpy
arrays.  It raises if the library has not been built -- there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libftattn.so")

F16, BF16, F32 = 0, 1, 2
ST_S, ST_EXP, ST_ROWSUM, ST_OACC = 0, 1, 2, 3
CHECK_S, CHECK_EXP, CHECK_L, CHECK_O = 0, 1, 2, 3
FT_OFF, FT_CORRECT, FT_DETECT = 0, 1, 2
OK, EINVAL, EUNSUPPORTED, EHIP, ENOMEM = 0, -1, -2, -3, -4
RANGE_OPERAND_OVERFLOW, RANGE_OPERAND_UNDERFLOW, RANGE_CHECKSUM_OVERFLOW = 1, 2, 4

EXPORTS = ("ftattn_create", "ftattn_get_config", "ftattn_forward", "ftattn_report", "ftattn_destroy",
           "ftattn_last_error", "ftattn_set_timing", "ftattn_get_timing", "ftattn_forward_static",
           "ftattn_static_last_error")
STATIC_SCRATCH_MIB = 64


class Config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("batch", C.c_int32), ("heads", C.c_int32), ("seq", C.c_int32),
                ("head_dim", C.c_int32), ("in_dtype", C.c_int32), ("out_dtype", C.c_int32), ("causal", C.c_int32),
                ("softmax_scale", C.c_float), ("ft_mode", C.c_int32), ("stride", C.c_int32), ("block_m", C.c_int32),
                ("block_n", C.c_int32), ("eps1", C.c_float), ("tau_o", C.c_float), ("delta_l", C.c_float),
                ("rowsum_fold", C.c_int32), ("per_step", C.c_int32), ("rescale_margin", C.c_float), ("max_events", C.c_int32),
                ("device", C.c_int32)]


class Fault(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("b", "h", "stage", "kv_tile", "row", "col", "bit")]


class Event(C.Structure):
    _fields_ = [("b", C.c_int32), ("h", C.c_int32), ("check", C.c_int32), ("kv_tile", C.c_int32), ("row", C.c_int32),
                ("col", C.c_int32), ("residual", C.c_float), ("action", C.c_int32)]


class ReportView(C.Structure):
    _fields_ = [("n_events", C.c_int32), ("n_events_dropped", C.c_int32), ("events", C.POINTER(Event)),
                ("tiles_m", C.c_int32), ("tiles_n", C.c_int32), ("tile_flags", C.POINTER(C.c_uint8)),
                ("rowtile_flags", C.POINTER(C.c_uint8)), ("residual_max", C.POINTER(C.c_float)),
                ("recheck_entries", C.c_int64), ("range_flags", C.c_int32)]


EVENT_DTYPE = np.dtype([("b", "<i4"), ("h", "<i4"), ("check", "<i4"), ("kv_tile", "<i4"), ("row", "<i4"),
                        ("col", "<i4"), ("residual", "<f4"), ("action", "<i4")])

_lib = None


class FtAttnError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"ftattn error {code}: {msg}")
        self.code = code


def load_library() -> C.CDLL:
    """Loads the built library; raises if it is missing (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_2504_02211_amd.build`")
    # The caller's tensors live in torch's HIP runtime; load that runtime first so that this
    # library binds to the same one instead of bringing a second copy into the process.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(LIB_PATH)
    lib.ftattn_create.argtypes = [C.POINTER(Config), C.POINTER(C.c_void_p)]
    lib.ftattn_get_config.argtypes = [C.c_void_p, C.POINTER(Config)]
    lib.ftattn_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(Fault),
                                   C.c_int32, C.c_void_p]
    lib.ftattn_report.argtypes = [C.c_void_p, C.POINTER(ReportView)]
    lib.ftattn_destroy.argtypes = [C.c_void_p]
    lib.ftattn_set_timing.argtypes = [C.c_void_p, C.c_int32]
    lib.ftattn_get_timing.argtypes = [C.c_void_p, C.POINTER(C.c_float)]
    lib.ftattn_last_error.argtypes = [C.c_void_p]
    lib.ftattn_last_error.restype = C.c_char_p
    lib.ftattn_forward_static.argtypes = [C.POINTER(Config), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_void_p]
    lib.ftattn_static_last_error.argtypes = []
    lib.ftattn_static_last_error.restype = C.c_char_p
    for n in ("ftattn_create", "ftattn_get_config", "ftattn_forward", "ftattn_report", "ftattn_destroy",
              "ftattn_set_timing", "ftattn_get_timing", "ftattn_forward_static"):
        getattr(lib, n).restype = C.c_int
    _lib = lib
    return lib


class Report:
    """Host copy of ftattn_report's view."""

    def __init__(self, view: ReportView, batch: int, heads: int):
        n = view.n_events
        self.n_events = n
        self.n_events_dropped = view.n_events_dropped
        self.tiles_m, self.tiles_n = view.tiles_m, view.tiles_n
        if n:
            buf = C.string_at(view.events, n * C.sizeof(Event))
            self.events = np.frombuffer(buf, dtype=EVENT_DTYPE).copy()
        else:
            self.events = np.zeros(0, dtype=EVENT_DTYPE)
        nrt = batch * heads * view.tiles_m
        self.tile_flags = np.ctypeslib.as_array(view.tile_flags, shape=(nrt * view.tiles_n,)).copy().reshape(
            batch, heads, view.tiles_m, view.tiles_n)
        self.rowtile_flags = np.ctypeslib.as_array(view.rowtile_flags, shape=(nrt,)).copy().reshape(
            batch, heads, view.tiles_m)
        self.residual_max = np.ctypeslib.as_array(view.residual_max, shape=(nrt * 4,)).copy().reshape(
            batch, heads, view.tiles_m, 4)
        self.recheck_entries = int(view.recheck_entries)
        self.range_flags = int(view.range_flags)

    def event_set(self):
        """Set of (b, h, check, kv_tile, row, col) tuples."""
        e = self.events
        return set(zip(e["b"].tolist(), e["h"].tolist(), e["check"].tolist(), e["kv_tile"].tolist(),
                       e["row"].tolist(), e["col"].tolist()))


_ITEMSIZE = {F16: 2, BF16: 2, F32: 4}
_TORCH_NAME = {F16: "torch.float16", BF16: "torch.bfloat16", F32: "torch.float32"}


def device_pointer(t, name: str, n_elems: int, dtype: int, device: int) -> C.c_void_p:
    """Address of a caller's tensor for the C ABI.  An integer is taken as a device address as it
    is; an object with the tensor protocol (torch) is checked first -- element type, element count,
    contiguity, device -- because the library can only see a raw pointer, and a tensor of the
    wrong size or type would turn into an out-of-bounds access on the GPU instead of an error."""
    if isinstance(t, int):
        return C.c_void_p(t)
    if not hasattr(t, "data_ptr"):
        raise TypeError(f"{name}: expected a device tensor or an integer address, got {type(t).__name__}")
    if hasattr(t, "is_cuda") and not t.is_cuda:
        raise ValueError(f"{name}: tensor is not on a GPU")
    if hasattr(t, "device") and getattr(t.device, "index", None) not in (None, device):
        raise ValueError(f"{name}: tensor is on device {t.device.index}, the context on device {device}")
    if hasattr(t, "is_contiguous") and not t.is_contiguous():
        raise ValueError(f"{name}: tensor is not contiguous")
    if hasattr(t, "dtype") and str(t.dtype) != _TORCH_NAME[dtype]:
        raise ValueError(f"{name}: tensor is {t.dtype}, expected {_TORCH_NAME[dtype]}")
    if hasattr(t, "numel") and t.numel() != n_elems:
        raise ValueError(f"{name}: tensor has {t.numel()} elements, the configured shape has {n_elems}")
    return C.c_void_p(t.data_ptr())


def forward_static(q, k, v, o, batch: int, heads: int, seq: int, head_dim: int, in_dtype: int, causal: bool,
                   out_dtype: int = F32, ft_mode: int = FT_CORRECT, softmax_scale: float = 0.0, n_events=None,
                   stream: int = 0, device: int = 0, rowsum_fold: bool = False) -> None:
    """ftattn_forward_static: one pass without a context and without any allocation, on the
    library's static scratch array.  n_events: a device int32 tensor (or address) that receives the
    number of events, or None."""
    lib = load_library()
    cfg = Config(C.sizeof(Config), batch, heads, seq, head_dim, in_dtype, out_dtype, int(bool(causal)), softmax_scale,
                 ft_mode, 8, 0, 0, 0.0, 0.0, 0.0, int(bool(rowsum_fold)), 0, 0.0, 0, device)
    n = batch * heads * seq * head_dim
    ptr = lambda t, name, dt: C.c_void_p(None) if t is None else device_pointer(t, name, n, dt, device)
    nev = C.c_void_p(None) if n_events is None else C.c_void_p(n_events if isinstance(n_events, int) else n_events.data_ptr())
    rc = lib.ftattn_forward_static(C.byref(cfg), ptr(q, "q", in_dtype), ptr(k, "k", in_dtype), ptr(v, "v", in_dtype),
                                   ptr(o, "o", out_dtype), nev, C.c_void_p(stream))
    if rc != OK:
        raise FtAttnError(rc, lib.ftattn_static_last_error().decode())


class FtAttn:
    """One context of the C library (one shape, one device)."""

    def __init__(self, batch: int, heads: int, seq: int, head_dim: int, in_dtype: int, causal: bool,
                 out_dtype: int = F32, ft_mode: int = FT_CORRECT, softmax_scale: float = 0.0, block_m: int = 0,
                 eps1: float = 0.0, tau_o: float = 0.0, delta_l: float = 0.0, max_events: int = 0, device: int = 0,
                 rowsum_fold: bool = False, per_step: int = 0, stride: int = 8, rescale_margin: float = 0.0):
        self.lib = load_library()
        cfg = Config(C.sizeof(Config), batch, heads, seq, head_dim, in_dtype, out_dtype, int(bool(causal)),
                     softmax_scale, ft_mode, int(stride), block_m, 0, eps1, tau_o, delta_l, int(bool(rowsum_fold)), int(per_step),
                     float(rescale_margin), max_events, device)
        self.handle = C.c_void_p()
        rc = self.lib.ftattn_create(C.byref(cfg), C.byref(self.handle))
        if rc != OK:
            self.handle = C.c_void_p()
            raise FtAttnError(rc, self.lib.ftattn_last_error(None).decode())
        eff = Config()
        self.lib.ftattn_get_config(self.handle, C.byref(eff))
        self.config = eff

    def forward(self, q, k, v, o, faults: Optional[np.ndarray] = None, stream: int = 0) -> None:
        """q, k, v, o: objects with data_ptr() (torch device tensors) or integer device addresses.
        faults: int32 array [n, 7] of (b, h, stage, kv_tile, row, col, bit)."""
        c = self.config
        ne = c.batch * c.heads * c.seq * c.head_dim
        ptr = lambda t, name, dt: device_pointer(t, name, ne, dt, c.device)
        n = 0
        fp = None
        if faults is not None and len(faults):
            fa = np.ascontiguousarray(faults, dtype=np.int32).reshape(-1, 7)
            n = fa.shape[0]
            fp = fa.ctypes.data_as(C.POINTER(Fault))
        rc = self.lib.ftattn_forward(self.handle, ptr(q, "q", c.in_dtype), ptr(k, "k", c.in_dtype), ptr(v, "v", c.in_dtype),
                                     ptr(o, "o", c.out_dtype), fp, n, C.c_void_p(stream))
        if rc != OK:
            raise FtAttnError(rc, self.lib.ftattn_last_error(self.handle).decode())

    def report(self) -> Report:
        view = ReportView()
        rc = self.lib.ftattn_report(self.handle, C.byref(view))
        if rc != OK:
            raise FtAttnError(rc, self.lib.ftattn_last_error(self.handle).decode())
        return Report(view, self.config.batch, self.config.heads)

    def set_timing(self, enabled: bool) -> None:
        rc = self.lib.ftattn_set_timing(self.handle, int(enabled))
        if rc != OK:
            raise FtAttnError(rc, self.lib.ftattn_last_error(self.handle).decode())

    def get_timing(self):
        """(encode ms, fused-kernel ms) of the last forward; needs set_timing(True)."""
        ms = (C.c_float * 2)()
        rc = self.lib.ftattn_get_timing(self.handle, ms)
        if rc != OK:
            raise FtAttnError(rc, self.lib.ftattn_last_error(self.handle).decode())
        return float(ms[0]), float(ms[1])

    def close(self) -> None:
        if self.handle:
            self.lib.ftattn_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
