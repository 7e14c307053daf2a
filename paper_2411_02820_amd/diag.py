"""ctypes binding of libdsk_diag.so (include/dsk_diag.h): device measurements for benchmarks, marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import torch  # noqa: F401  (first, so that the process ends up with one HIP runtime; see binding.py)

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdsk_diag.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2411_02820_amd.build)")

lib = C.CDLL(LIB_PATH)
lib.dsk_diag_mfma_peak.argtypes = [C.POINTER(C.c_double), C.c_void_p]
lib.dsk_diag_mfma_peak.restype = C.c_int

EXPORTS = ("dsk_diag_mfma_peak",)


def dsk_diag_mfma_peak(stream=None) -> float:
    out = C.c_double(0.0)
    rc = lib.dsk_diag_mfma_peak(C.byref(out), None if stream is None else stream.cuda_stream)
    if rc != 0:
        raise RuntimeError(f"dsk_diag_mfma_peak failed [{rc}]")
    return out.value
