"""ctypes binding of libhfr_probe (include/hfr_probe.h): the benchmark's
streaming probes. Argument marshalling only; not part of the reduction path."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhfr_probe.so")

HFR_PROBE_WIDE = 0
HFR_PROBE_BULK = 1
HFR_PROBE_MAX_STREAMS = 16

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libhfr_probe.so is not built: run `python -m paper_2408_14158_amd.build`")
        try:
            import torch  # noqa: F401  (one HIP runtime instance, as for libhfr)
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        L.hfr_probe_stream.argtypes = [ctypes.POINTER(vp), ctypes.c_int, ctypes.POINTER(vp), ctypes.c_int, vp,
                                       ctypes.c_size_t, ctypes.c_int, vp]
        L.hfr_probe_stream.restype = ctypes.c_int
        L.hfr_probe_stream_paced.argtypes = [ctypes.POINTER(vp), ctypes.c_int, ctypes.POINTER(vp), ctypes.c_int, vp,
                                             ctypes.c_size_t, ctypes.c_int, ctypes.c_int, vp]
        L.hfr_probe_stream_paced.restype = ctypes.c_int
        _lib = L
    return _lib


def _addr(x) -> int:
    return 0 if x is None else (x if isinstance(x, int) else int(x.data_ptr()))


def hfr_probe_stream(rd, wr, sink, nbytes: int, shape: int, stream=None, check: bool = True) -> int:
    """One streaming pass over nbytes: len(rd) read streams, len(wr) write streams."""
    rd, wr = list(rd or []), list(wr or [])
    ra = (ctypes.c_void_p * max(len(rd), 1))(*[_addr(p) for p in rd])
    wa = (ctypes.c_void_p * max(len(wr), 1))(*[_addr(p) for p in wr])
    s = 0 if stream is None else (stream if isinstance(stream, int) else int(stream.cuda_stream))
    st = lib().hfr_probe_stream(ra, len(rd), wa, len(wr), _addr(sink), int(nbytes), int(shape), s)
    if check and st != 0:
        raise RuntimeError("hfr_probe_stream failed with status %d" % st)
    return st


def hfr_probe_stream_paced(rd, wr, sink, nbytes: int, lanes: int, pace: int, stream=None, check: bool = True) -> int:
    """The bulk shape with `lanes` per workgroup and a pause of pace * 64 clocks after each trip."""
    rd, wr = list(rd or []), list(wr or [])
    ra = (ctypes.c_void_p * max(len(rd), 1))(*[_addr(p) for p in rd])
    wa = (ctypes.c_void_p * max(len(wr), 1))(*[_addr(p) for p in wr])
    s = 0 if stream is None else (stream if isinstance(stream, int) else int(stream.cuda_stream))
    st = lib().hfr_probe_stream_paced(ra, len(rd), wa, len(wr), _addr(sink), int(nbytes), int(lanes), int(pace), s)
    if check and st != 0:
        raise RuntimeError("hfr_probe_stream_paced failed with status %d" % st)
    return st
