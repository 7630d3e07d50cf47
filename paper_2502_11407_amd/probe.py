"""ctypes face of libgensor_probe.so: the benchmark's MFMA-only probe kernel (csrc/probe.cpp), a
measurement aid that is not part of the operator library.  Marshalling only."""
from __future__ import annotations

import ctypes as C
import os

from .binding import DTYPE, GensorError, _stream_ptr

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libgensor_probe.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2502_11407_amd.csrc.build`")
_lib = C.CDLL(LIB_PATH)
_lib.gensor_probe_mfma.restype = C.c_int
_lib.gensor_probe_mfma.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]


def mfma_probe(dtype: str, operands, sink, iters: int, workgroups: int, stream=None):
    """`workgroups` workgroups of 4 wavefronts run `iters` rounds of 8 MFMAs on the fragments in `operands`
    (a 256 KiB device tensor); `sink` is a device tensor of workgroups * 256 floats."""
    st = _lib.gensor_probe_mfma(DTYPE[dtype], operands.data_ptr(), sink.data_ptr(), iters, workgroups, _stream_ptr(stream))
    if st != 0:
        raise GensorError(st, "gensor_probe_mfma")
