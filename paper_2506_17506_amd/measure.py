"""ctypes binding of the benchmark's measurement hooks (include/vl_bench.h).  Not part of
the verifier's interface: bench.py uses them, nothing else needs them."""
from __future__ import annotations

import ctypes as C
import os

from . import binding

BENCH_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libvlbench.so")
_bench = None


def _bench_lib():
    global _bench
    if _bench is None:
        if not os.path.exists(BENCH_LIB_PATH):
            raise RuntimeError(f"{BENCH_LIB_PATH} is missing: build it with `python -m paper_2506_17506_amd.build`")
        binding.load()   # torch and the HIP runtime first
        L = C.CDLL(BENCH_LIB_PATH)
        L.vl_stream_read_probe.restype = C.c_int32
        L.vl_stream_read_probe.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]
        _bench = L
    return _bench


def vl_stream_read_probe(buf, n_bytes: int, sink, stream=None) -> int:
    """One launch that reads n_bytes of buf; returns the hook's code (0 = launched)."""
    return int(_bench_lib().vl_stream_read_probe(C.c_void_p(binding._dev_ptr(buf)), n_bytes,
                                                 C.c_void_p(binding._dev_ptr(sink)), binding._stream_ptr(stream)))


def vl_verify_time_next(start_event, stop_event) -> None:
    """start_event / stop_event: raw hipEvent_t handles (ints) or None; recorded around the
    candidate-walk kernel of the next verification call on this thread."""
    L = binding.load()
    L.vl_verify_time_next.restype = C.c_int32
    L.vl_verify_time_next.argtypes = [C.c_void_p, C.c_void_p]
    L.vl_verify_time_next(C.c_void_p(start_event), C.c_void_p(stop_event))
