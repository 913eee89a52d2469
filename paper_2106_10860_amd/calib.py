"""Loader of libmaddness_calib.so: a plain device copy kernel of known traffic.

Not part of the method and not part of libmaddness; ``bench.py`` uses it to quote a copy
rate beside its own figures and to scale the profiler's memory counters.
"""
from __future__ import annotations

import ctypes as C
import os

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmaddness_calib.so")
_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: run `python -m paper_2106_10860_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.calib_stream_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        _lib = L
    return _lib


def stream_copy(src, dst, stream=None) -> None:
    """Copies the bytes of device tensor ``src`` to ``dst`` (same size) with the plain copy kernel."""
    import torch
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("src and dst differ in size")
    s = torch.cuda.current_stream() if stream is None else stream
    rc = lib().calib_stream_copy(src.data_ptr(), dst.data_ptr(), nbytes, s.cuda_stream or None)
    if rc != 0:
        raise RuntimeError(f"calib_stream_copy failed with status {rc}")
