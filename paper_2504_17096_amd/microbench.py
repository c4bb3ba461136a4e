"""ctypes binding of libsailor_microbench.so (include/sailor_microbench.h): the FMA-chain and
write kernels that calibrate the benchmark's rooflines.  Marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsailor_microbench.so")
EXPORTS = ["sailor_microbench_fma", "sailor_microbench_write", "sailor_microbench_write_records"]
_lib = None


def load_library() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with "
                              "`python -m paper_2504_17096_amd.build` (hipcc, gfx950)")
        lib = C.CDLL(LIB_PATH)
        lib.sailor_microbench_fma.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_double),
                                              C.POINTER(C.c_double), C.c_void_p]
        lib.sailor_microbench_write.argtypes = [C.c_uint64, C.c_int32, C.POINTER(C.c_double),
                                                C.POINTER(C.c_double), C.c_void_p]
        lib.sailor_microbench_write_records.argtypes = [C.c_uint64, C.c_int32, C.POINTER(C.c_double),
                                                        C.POINTER(C.c_double), C.c_void_p]
        for name in EXPORTS:
            getattr(lib, name).restype = C.c_int
        _lib = lib
    return _lib


def fma(workgroups: int = 256 * 8, iters: int = 4096, reps: int = 5, stream: int = 0) -> Tuple[float, float]:
    """(TFLOP/s, ms of the fastest repetition) of the FMA chain."""
    t, ms = C.c_double(), C.c_double()
    rc = load_library().sailor_microbench_fma(workgroups, iters, reps, C.byref(t), C.byref(ms),
                                              stream or None)
    if rc != 0:
        raise RuntimeError(f"sailor_microbench_fma: {rc}")
    return t.value, ms.value


def write(nbytes: int = 1 << 31, reps: int = 5, stream: int = 0) -> Tuple[float, float]:
    """(1e9 bytes/s, ms of the fastest repetition) of the streaming store."""
    g, ms = C.c_double(), C.c_double()
    rc = load_library().sailor_microbench_write(nbytes, reps, C.byref(g), C.byref(ms), stream or None)
    if rc != 0:
        raise RuntimeError(f"sailor_microbench_write: {rc}")
    return g.value, ms.value


def write_records(elements: int = 104_256_000, reps: int = 5, stream: int = 0) -> Tuple[float, float]:
    """(1e9 bytes/s, ms of the fastest repetition) of writing four arrays of 4 + 4 + 8 + 4 bytes
    per element, the output format of the per-candidate evaluation."""
    g, ms = C.c_double(), C.c_double()
    rc = load_library().sailor_microbench_write_records(elements, reps, C.byref(g), C.byref(ms), stream or None)
    if rc != 0:
        raise RuntimeError(f"sailor_microbench_write_records: {rc}")
    return g.value, ms.value
