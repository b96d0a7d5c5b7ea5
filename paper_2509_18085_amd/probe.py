"""ctypes binding of libspiffy_probe.so (include/spiffy_probe.h): the two machine microbenchmarks behind the measured
peaks of bench.py.  Separate from the verification library on purpose: nothing on the product path loads this."""
from __future__ import annotations

import ctypes as C
import os

import torch

from .spiffy import SpiffyError, _ptr, _stream

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libspiffy_probe.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libspiffy_probe.so is not built (%s missing): run `python -m paper_2509_18085_amd.build`" % LIB_PATH)
lib = C.CDLL(LIB_PATH)
lib.spiffy_probe_mfma.restype = C.c_int
lib.spiffy_probe_mfma.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]
lib.spiffy_probe_hbm_read.restype = C.c_int
lib.spiffy_probe_hbm_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]


def probe_mfma(iters: int, random_operands: bool, sink: torch.Tensor, stream=None) -> float:
    """Launch the register-only MFMA loop; returns the flop of the launch (time it with events)."""
    flop = C.c_double(0.0)
    rc = lib.spiffy_probe_mfma(iters, 1 if random_operands else 0, _ptr(sink), C.byref(flop), _stream(stream))
    if rc:
        raise SpiffyError(rc, "spiffy_probe_mfma")
    return flop.value


def probe_hbm_read(src: torch.Tensor, sink: torch.Tensor, stream=None) -> int:
    """Launch one read-only pass over src; returns the bytes read."""
    n = src.numel() * src.element_size()
    rc = lib.spiffy_probe_hbm_read(_ptr(src), n, _ptr(sink), _stream(stream))
    if rc:
        raise SpiffyError(rc, "spiffy_probe_hbm_read")
    return n
