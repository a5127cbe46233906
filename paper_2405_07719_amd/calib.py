"""Binding of the matrix-core calibration loops (libusp_calib.so): a measurement aid that bench.py reports next
to the forward kernel's roofline fraction.  Not part of the product library or its ABI."""
from __future__ import annotations

import ctypes as C
import os

from . import UspError, USP_OK, _ptr, _stream

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libusp_calib.so")
USP_CALIB_SINK_BYTES = 256 * 512 * 4
_lib = None


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2405_07719_amd.build`")
        import torch  # noqa: F401  (first: the process must hold ONE HIP runtime, the one torch ships)
        lib = C.CDLL(LIB_PATH)
        lib.usp_calib_mfma.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.POINTER(C.c_double), C.c_void_p]
        lib.usp_calib_mfma.restype = C.c_int
        _lib = lib
    return _lib


def usp_calib_mfma(mode, iters, sink, stream=None):
    """Enqueue one calibration launch (0 pure MFMA, 1 attention mix); returns its MFMA flop count."""
    flop = C.c_double(0.0)
    st = load().usp_calib_mfma(mode, iters, _ptr(sink), sink.numel() * sink.element_size(), C.byref(flop), _stream(stream))
    if st != USP_OK:
        raise UspError(st, "usp_calib_mfma")
    return flop.value
