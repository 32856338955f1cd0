"""ctypes binding of libdos_probe.so: the benchmark's measurement aids (see
probe/dos_probe.h).  Not part of the product path; bench.py loads it for its
ceiling measurements and for the known-size copy kernel that scales hardware
traffic counters."""
from __future__ import annotations

import ctypes as C
import os

from . import binding as _b

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdos_probe.so")
DEFAULT_LDS_CAP = 14848      # DOS_PROBE_DEFAULT_LDS_CAP

_lib = None


def load():
    global _lib
    if _lib is None:
        _b.load()                                  # torch's HIP runtime first, as for libdos
        lib = C.CDLL(LIB_PATH)
        lib.dos_probe_copy.restype = C.c_int
        lib.dos_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
        lib.dos_probe_adam_traffic.restype = C.c_int
        lib.dos_probe_adam_traffic.argtypes = [C.POINTER(_b.dos_subgroup), C.c_int32, C.c_int32, C.c_void_p]
        lib.dos_probe_host_stream.restype = C.c_int
        lib.dos_probe_host_stream.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64,
                                              C.c_uint64, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_double)]
        _lib = lib
    return _lib


def dos_probe_copy(dst: int, src: int, nbytes: int, stream: int = 0) -> None:
    _b.check(load().dos_probe_copy(C.c_void_p(dst), C.c_void_p(src), int(nbytes), C.c_void_p(stream)), "dos_probe_copy")


def dos_probe_adam_traffic(sg, mode: int, stream: int = 0, lds_bytes: int = 0) -> None:
    _b.check(load().dos_probe_adam_traffic(C.byref(sg), int(mode), int(lds_bytes), C.c_void_p(stream)),
             "dos_probe_adam_traffic")


def dos_probe_host_stream(p: int, m: int, v: int, g: int, out16: int, n: int, out_n: int, threads: int, reps: int,
                          streamed: bool) -> float:
    """Seconds for `reps` sweeps of the host update's access pattern over n elements."""
    sec = C.c_double()
    _b.check(load().dos_probe_host_stream(C.c_void_p(p), C.c_void_p(m), C.c_void_p(v), C.c_void_p(g), C.c_void_p(out16),
                                          int(n), int(out_n), int(threads), int(reps), int(streamed),
                                          C.byref(sec)), "dos_probe_host_stream")
    return sec.value
