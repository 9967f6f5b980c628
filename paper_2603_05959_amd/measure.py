"""ctypes binding of libovggt_measure.so (include/ovggt_measure.h): the MFMA-loop rate that
bench.py reports beside the published peak.  Not part of the hot path."""
from __future__ import annotations

import ctypes as C
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libovggt_measure.so")
EXPORTS = ("ovggt_measure_mfma_loop",)

_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2603_05959_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.ovggt_measure_mfma_loop.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_double), C.c_void_p]
        L.ovggt_measure_mfma_loop.restype = C.c_int
        _lib = L
    return _lib


def ovggt_measure_mfma_loop(sink, workgroups: int, random_operands: bool, iters: int = 20000, stream: int = 0) -> float:
    """TFLOP/s; `sink` is a torch device tensor (or a device address) of at least 4 bytes."""
    v = C.c_double()
    ptr = sink if isinstance(sink, int) or sink is None else sink.data_ptr()
    code = lib().ovggt_measure_mfma_loop(ptr, workgroups, 1 if random_operands else 0, iters, C.byref(v), stream)
    if code != 0:
        raise RuntimeError(f"ovggt_measure_mfma_loop: error {code}")
    return float(v.value)
