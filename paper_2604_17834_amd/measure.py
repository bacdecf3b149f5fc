"""ctypes binding of libasyncsparse_measure.so: the benchmark's two probe kernels (matrix-core rate, read-only
stream).  Measurement support only -- not part of the product library, nothing of the method runs here."""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libasyncsparse_measure.so")
EXPORTED_SYMBOLS = ["asp_probe_mfma", "asp_probe_read"]
_DT = {"bf16": 0, "f32": 1}
_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libasyncsparse_measure.so is missing: build it with `python -m paper_2604_17834_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64 = ctypes.c_void_p, ctypes.c_int64
        L.asp_probe_mfma.argtypes = [ctypes.c_int32, i64, vp, vp, ctypes.POINTER(ctypes.c_double)]
        L.asp_probe_mfma.restype = ctypes.c_int
        L.asp_probe_read.argtypes = [vp, i64, vp, vp]
        L.asp_probe_read.restype = ctypes.c_int
        _lib = L
    return _lib


def asp_probe_mfma(dtype, iters, out_ptr, stream=None) -> float:
    """Enqueue the matrix-core-only kernel; returns the number of floating-point operations it performs."""
    flop = ctypes.c_double()
    st = lib().asp_probe_mfma(_DT.get(dtype, dtype), iters, out_ptr, stream, ctypes.byref(flop))
    if st != 0:
        raise RuntimeError("asp_probe_mfma: status %d" % st)
    return flop.value


def asp_probe_read(src_ptr, nbytes, out_ptr, stream=None):
    """Enqueue the read-only stream kernel over nbytes of device memory."""
    st = lib().asp_probe_read(src_ptr, nbytes, out_ptr, stream)
    if st != 0:
        raise RuntimeError("asp_probe_read: status %d" % st)
    return st
