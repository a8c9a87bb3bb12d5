"""ctypes binding of libhfr: the same names and argument order as the C ABI
(include/hfr.h). Argument marshalling only - every step runs in the library's
HIP kernels. There is no fallback: if the shared library is missing, loading
fails loudly.

Buffers may be passed as integer device addresses or as torch tensors (their
``data_ptr()`` is taken; dtype and contiguity are the caller's business, as in
C). ``stream`` is a raw hipStream_t handle as an int (``torch.cuda.Stream
.cuda_stream``), a torch stream object, or None / 0 for the null stream.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhfr.so")

HFR_OK = 0
HFR_ERR_INVALID_ARG = 1
HFR_ERR_UNSUPPORTED_DTYPE = 2
HFR_ERR_MISALIGNED = 3
HFR_ERR_OVERLAP = 4
HFR_ERR_HIP = 5

HFR_F32 = 0
HFR_BF16 = 1
HFR_F16 = 2
HFR_FP8_E4M3 = 3
HFR_FP8_E5M2 = 4

HFR_MAX_K = 16
HFR_MAX_STREAMS = 16
HFR_NOALLOC_MAX_CHUNKS = 4096

HFR_TUNE_GRID_CAP = 0
HFR_TUNE_UNROLL = 1
HFR_TUNE_BULK_GRID = 2
HFR_TUNE_BULK_MIN_BYTES = 3
HFR_TUNE_BULK_SKEW = 4
HFR_TUNE_BUCKET_FOLD = 5
HFR_TUNE_PLACEMENT_ONLINE = 6
HFR_TUNE_SEGMENT_MIB = 7
HFR_TUNE_BULK_BLOCK = 8
HFR_TUNE_BULK_PACE = 9
HFR_TUNE_WIDE_WGS_PER_CU = 10
HFR_TUNE_BUCKET_LIST = 11

ELEM_SIZE = {HFR_F32: 4, HFR_BF16: 2, HFR_F16: 2, HFR_FP8_E4M3: 1, HFR_FP8_E5M2: 1}


class HfrError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("libhfr: %s (status %d)" % (text, status))
        self.status = status


class hfr_bucket(ctypes.Structure):
    _fields_ = [("in_", ctypes.POINTER(ctypes.c_void_p)), ("out", ctypes.c_void_p),
                ("n", ctypes.c_size_t)]


_lib = None


def _check_single_hip_runtime():
    """Two HIP runtimes in one process cannot see each other's memory or
    streams; refuse to go on if that happened."""
    try:
        with open("/proc/self/maps") as f:
            paths = {line.split()[-1] for line in f if "libamdhip64" in line}
    except OSError:
        return
    real = {os.path.realpath(p) for p in paths}
    if len(real) > 1:
        raise ImportError("two HIP runtimes are loaded (%s): import torch before "
                          "paper_2408_14158_amd.hfr" % ", ".join(sorted(real)))


def lib() -> ctypes.CDLL:
    """The loaded shared library (loads it on first use)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "libhfr.so is not built: run `python -m paper_2408_14158_amd.build` "
                "(there is no CPU fallback)")
        # Device pointers and streams handed to the library come from PyTorch, so
        # both must run on ONE HIP runtime instance. PyTorch ships its own
        # libamdhip64 (soname libamdhip64.so.7); importing torch first makes the
        # dynamic loader resolve libhfr's dependency to that already-loaded copy.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        _check_single_hip_runtime()
        vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        L.hfr_reduce_sum.argtypes = [ctypes.POINTER(vp), ci, vp, sz, ci, vp]
        L.hfr_reduce_sum.restype = ci
        L.hfr_combine_avg.argtypes = [vp, vp, vp, sz, ctypes.c_float, ci, vp]
        L.hfr_combine_avg.restype = ci
        L.hfr_reduce_avg.argtypes = [ctypes.POINTER(vp), ci, vp, sz, ctypes.c_float, ci, vp]
        L.hfr_reduce_avg.restype = ci
        L.hfr_reduce_combine_avg.argtypes = [ctypes.POINTER(vp), ci, vp, vp, sz, ctypes.c_float, ci, vp]
        L.hfr_reduce_combine_avg.restype = ci
        L.hfr_reduce_scatter_slice.argtypes = [ctypes.POINTER(vp), ci, vp, sz, ci, ci, ci, vp]
        L.hfr_reduce_scatter_slice.restype = ci
        L.hfr_slice_bounds.argtypes = [sz, ci, ci, ctypes.POINTER(sz), ctypes.POINTER(sz)]
        L.hfr_slice_bounds.restype = None
        L.hfr_broadcast.argtypes = [vp, ctypes.POINTER(vp), ci, sz, ci, vp]
        L.hfr_broadcast.restype = ci
        L.hfr_reduce_buckets.argtypes = [ctypes.POINTER(hfr_bucket), sz, ci, ci, sz, ci, vp]
        L.hfr_reduce_buckets.restype = ci
        L.hfr_reduce_buckets_batched.argtypes = [ctypes.POINTER(hfr_bucket), sz, ci, ci, vp]
        L.hfr_reduce_buckets_batched.restype = ci
        L.hfr_init.argtypes = []
        L.hfr_init.restype = ci
        L.hfr_shutdown.argtypes = []
        L.hfr_shutdown.restype = ci
        L.hfr_status_string.argtypes = [ci]
        L.hfr_status_string.restype = ctypes.c_char_p
        L.hfr_last_error.argtypes = []
        L.hfr_last_error.restype = ctypes.c_char_p
        L.hfr_version.argtypes = []
        L.hfr_version.restype = ci
        L.hfr_reduce_chunk_table.argtypes = [vp, sz, sz, ci, ci, vp]
        L.hfr_reduce_chunk_table.restype = ci
        L.hfr_reduce_chunks_noalloc.argtypes = [vp, sz, sz, ci, ci, vp]
        L.hfr_reduce_chunks_noalloc.restype = ci
        L.hfr_tune_placement.argtypes = [ctypes.POINTER(vp), ci, vp, sz, ci, vp, ctypes.POINTER(ci)]
        L.hfr_tune_placement.restype = ci
        L.hfr_placement_query.argtypes = [ctypes.POINTER(vp), ci, vp, ci, ctypes.POINTER(ci), ctypes.POINTER(ci)]
        L.hfr_placement_query.restype = ci
        L.hfr_device_info.argtypes = [ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(ci)]
        L.hfr_device_info.restype = ci
        L.hfr_peer_stride.argtypes = [ctypes.c_size_t]
        L.hfr_peer_stride.restype = ctypes.c_size_t
        L.hfr_tune_peer_stride.argtypes = [vp, sz, ci, sz, ci, vp, ctypes.POINTER(ctypes.c_size_t)]
        L.hfr_tune_peer_stride.restype = ci
        L.hfr_set_tuning.argtypes = [ci, ctypes.c_long]
        L.hfr_set_tuning.restype = ci
        _lib = L
    return _lib


def _ptr(x) -> int:
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _ptr_array(ptrs, K, what="in"):
    """HOST array of device pointers for a K-way call. The library reads K
    entries, so a list shorter than K is refused here (it would read past the
    end of the array)."""
    if ptrs is None:
        return None
    if len(ptrs) < int(K) <= HFR_MAX_K:     # a K the library rejects is never used as a length
        raise ValueError("%s holds %d pointers but K = %d" % (what, len(ptrs), int(K)))
    return (ctypes.c_void_p * max(len(ptrs), 1))(*[_ptr(p) for p in ptrs])


def _stream(s) -> int:
    if s is None:
        return 0
    if isinstance(s, int):
        return s
    return int(s.cuda_stream)


def _raise(status: int):
    L = lib()
    text = L.hfr_status_string(status).decode()
    if status == HFR_ERR_HIP:
        text += ": " + L.hfr_last_error().decode()
    raise HfrError(status, text)


def hfr_status_string(status: int) -> str:
    return lib().hfr_status_string(int(status)).decode()


def hfr_last_error() -> str:
    return lib().hfr_last_error().decode()


def hfr_version() -> int:
    return int(lib().hfr_version())


def hfr_device_info(check: bool = True):
    """(compute units, memory clock in kHz, memory bus width in bits) of the current device."""
    cu, clk, bus = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0)
    st = int(lib().hfr_device_info(ctypes.byref(cu), ctypes.byref(clk), ctypes.byref(bus)))
    if st != HFR_OK and check:
        _raise(st)
    return cu.value, clk.value, bus.value


def hfr_peer_stride(bytes_per_buffer: int) -> int:
    """Distance in bytes at which to carve the K inputs and the output from one allocation; see include/hfr.h."""
    return int(lib().hfr_peer_stride(int(bytes_per_buffer)))


def hfr_tune_peer_stride(arena, arena_bytes: int, K: int, n: int, dt: int, stream=None, check: bool = True):
    """Times candidate distances for K + 1 buffers of n elements inside `arena` (blocks the host,
    overwrites parts of the arena); returns (status, stride in bytes). See include/hfr.h."""
    stride = ctypes.c_size_t(0)
    st = lib().hfr_tune_peer_stride(_ptr(arena), int(arena_bytes), int(K), int(n), int(dt), _stream(stream),
                                    ctypes.byref(stride))
    if check and st != HFR_OK:
        _raise(st)
    return st, int(stride.value)


def hfr_reduce_sum(in_, K: int, out, n: int, dt: int, stream=None, check: bool = True) -> int:
    """out[i] = ((in_[0][i] + in_[1][i]) + ...) + in_[K-1][i]; see include/hfr.h."""
    arr = _ptr_array(in_, K)
    st = lib().hfr_reduce_sum(arr, int(K), _ptr(out), int(n), int(dt), _stream(stream))
    if check and st != HFR_OK:
        _raise(st)
    return st


CHUNK_ENTRY_WORDS = HFR_MAX_K + 2   # 8-byte words of one hfr_chunk: 16 input pointers, out, n


def make_chunk_table(chunks, device="cuda"):
    """Device tensor holding an hfr_chunk array for a list of (inputs, out, n)
    tuples of device tensors (argument marshalling: pointers and sizes only)."""
    import numpy as np
    import torch
    tab = np.zeros((max(len(chunks), 1), CHUNK_ENTRY_WORDS), dtype=np.uint64)
    for c, (ins, out, n) in enumerate(chunks):
        for j, t in enumerate(ins):
            tab[c, j] = _ptr(t)
        tab[c, HFR_MAX_K] = _ptr(out)
        tab[c, HFR_MAX_K + 1] = int(n)
    return torch.from_numpy(tab.view(np.int64)).to(device)


def make_host_chunk_array(chunks):
    """HOST hfr_chunk array (as a numpy uint64 matrix, one row per chunk) for a
    list of (inputs, out, n) tuples of device tensors or addresses."""
    import numpy as np
    tab = np.zeros((max(len(chunks), 1), CHUNK_ENTRY_WORDS), dtype=np.uint64)
    for c, (ins, out, n) in enumerate(chunks):
        for j, t in enumerate(ins):
            tab[c, j] = _ptr(t)
        tab[c, HFR_MAX_K] = _ptr(out)
        tab[c, HFR_MAX_K + 1] = int(n)
    return tab


def hfr_reduce_chunks_noalloc(chunks, n_chunks: int, chunk_elems_hint: int, K: int, dt: int, stream=None,
                              check: bool = True) -> int:
    """hfr_reduce_chunk_table with the chunk list on the HOST (a matrix from
    make_host_chunk_array, or None) and the device table in the library's
    static array: no allocation; see include/hfr.h."""
    addr = 0 if chunks is None else int(chunks.ctypes.data)
    st = lib().hfr_reduce_chunks_noalloc(addr, int(n_chunks), int(chunk_elems_hint), int(K), int(dt),
                                         _stream(stream))
    if check and st != HFR_OK:
        _raise(st)
    return st


def hfr_reduce_chunk_table(table, n_chunks: int, chunk_elems_hint: int, K: int, dt: int, stream=None,
                           check: bool = True) -> int:
    """K-way sum of every chunk of a table in device memory, one launch; see include/hfr.h."""
    st = lib().hfr_reduce_chunk_table(_ptr(table), int(n_chunks), int(chunk_elems_hint), int(K), int(dt),
                                      _stream(stream))
    if check and st != HFR_OK:
        _raise(st)
    return st


def hfr_tune_placement(in_, K: int, out, n: int, dt: int, stream=None, check: bool = True):
    """Times the plain and the skewed bulk kernels on these buffers and records
    the fastest for their placement (blocks the host); returns (status, pattern)."""
    arr = _ptr_array(in_, K)
    chosen = ctypes.c_int(0)
    st = lib().hfr_tune_placement(arr, int(K), _ptr(out), int(n), int(dt), _stream(stream), ctypes.byref(chosen))
    if check and st != HFR_OK:
        _raise(st)
    return st, chosen.value


def hfr_placement_query(in_, K: int, out, dt: int, check: bool = True):
    """(status, state, pattern) of the placement table for these buffers:
    state 0 unknown, 1 being measured, 2 recorded."""
    arr = _ptr_array(in_, K)
    state, pattern = ctypes.c_int(0), ctypes.c_int(0)
    st = lib().hfr_placement_query(arr, int(K), _ptr(out), int(dt), ctypes.byref(state), ctypes.byref(pattern))
    if check and st != HFR_OK:
        _raise(st)
    return st, state.value, pattern.value


def hfr_reduce_avg(in_, K: int, out, n: int, scale: float, dt: int, stream=None, check: bool = True) -> int:
    """out[i] = narrow(fl(in-order K-way fp32 sum * scale)); see include/hfr.h."""
    arr = _ptr_array(in_, K)
    st = lib().hfr_reduce_avg(arr, int(K), _ptr(out), int(n), ctypes.c_float(scale), int(dt), _stream(stream))
    if check and st != HFR_OK:
        _raise(st)
    return st


def hfr_reduce_combine_avg(in_, K: int, remote, out, n: int, scale: float, dt: int, stream=None,
                           check: bool = True) -> int:
    """hfr_reduce_sum then hfr_combine_avg with `remote`, in one kernel; see include/hfr.h."""
    arr = _ptr_array(in_, K)
    st = lib().hfr_reduce_combine_avg(arr, int(K), _ptr(remote), _ptr(out), int(n), ctypes.c_float(scale),
                                      int(dt), _stream(stream))
    if check and st != HFR_OK:
        _raise(st)
    return st


def hfr_reduce_scatter_slice(in_, K: int, out, n: int, rank: int, world: int, dt: int, stream=None,
                             check: bool = True) -> int:
    """K-way sum of slice `rank` of `world` only, written in place into the full out buffer."""
    arr = _ptr_array(in_, K)
    st = lib().hfr_reduce_scatter_slice(arr, int(K), _ptr(out), int(n), int(rank), int(world), int(dt),
                                        _stream(stream))
    if check and st != HFR_OK:
        _raise(st)
    return st


def hfr_slice_bounds(n: int, rank: int, world: int):
    """[begin, end) of slice `rank`; host-only arithmetic."""
    b, e = ctypes.c_size_t(), ctypes.c_size_t()
    lib().hfr_slice_bounds(int(n), int(rank), int(world), ctypes.byref(b), ctypes.byref(e))
    return int(b.value), int(e.value)


def hfr_broadcast(src, dst, K: int, n: int, dt: int, stream=None, check: bool = True) -> int:
    """dst[j][i] = src[i] for every j (one read, K writes); see include/hfr.h."""
    arr = _ptr_array(dst, K, "dst")
    st = lib().hfr_broadcast(_ptr(src), arr, int(K), int(n), int(dt), _stream(stream))
    if check and st != HFR_OK:
        _raise(st)
    return st


def hfr_combine_avg(a, b, out, n: int, scale: float, dt: int, stream=None, check: bool = True) -> int:
    """out[i] = fl(fl(a[i] + b[i]) * scale); see include/hfr.h."""
    st = lib().hfr_combine_avg(_ptr(a), _ptr(b), _ptr(out), int(n), ctypes.c_float(scale), int(dt),
                               _stream(stream))
    if check and st != HFR_OK:
        _raise(st)
    return st


def make_bucket_array(buckets, K=None):
    """Marshals [(ins, out, n), ...] into a C hfr_bucket array. Returns
    (array, keepalive); hold on to both for as long as the array is used.
    With K given, a bucket that lists fewer than K inputs is refused."""
    arr = (hfr_bucket * max(len(buckets), 1))()
    keep = []
    for i, (ins, out, n) in enumerate(buckets):
        if ins is None:
            arr[i].in_ = None
        else:
            if K is not None and len(ins) < int(K) <= HFR_MAX_K:
                raise ValueError("bucket %d holds %d pointers but K = %d" % (i, len(ins), int(K)))
            tab = (ctypes.c_void_p * max(len(ins), 1))(*[_ptr(p) for p in ins])
            keep.append(tab)
            arr[i].in_ = ctypes.cast(tab, ctypes.POINTER(ctypes.c_void_p))
        arr[i].out = _ptr(out)
        arr[i].n = int(n)
    return arr, keep


def hfr_reduce_buckets(buckets, n_buckets: int, K: int, dt: int, chunk_elems: int, n_streams: int,
                       stream=None, check: bool = True) -> int:
    """Chunked, stream-pipelined K-way sum over a bucket list; see include/hfr.h.

    ``buckets`` is a list of (ins, out, n) triples, or an array made by
    ``make_bucket_array`` (pass the (array, keepalive) pair as is)."""
    if isinstance(buckets, tuple) and len(buckets) == 2 and isinstance(buckets[0], ctypes.Array):
        arr, _keep = buckets
    elif buckets is None:
        arr, _keep = None, None
    else:
        arr, _keep = make_bucket_array(buckets, K)
    st = lib().hfr_reduce_buckets(arr, int(n_buckets), int(K), int(dt), int(chunk_elems),
                                  int(n_streams), _stream(stream))
    if check and st != HFR_OK:
        _raise(st)
    return st


def hfr_reduce_buckets_batched(buckets, n_buckets: int, K: int, dt: int, stream=None, check: bool = True) -> int:
    """Bucket-list reduction with small buckets folded into batched launches; see include/hfr.h."""
    if isinstance(buckets, tuple) and len(buckets) == 2 and isinstance(buckets[0], ctypes.Array):
        arr, _keep = buckets
    elif buckets is None:
        arr, _keep = None, None
    else:
        arr, _keep = make_bucket_array(buckets, K)
    st = lib().hfr_reduce_buckets_batched(arr, int(n_buckets), int(K), int(dt), _stream(stream))
    if check and st != HFR_OK:
        _raise(st)
    return st


def hfr_init(check: bool = True) -> int:
    st = lib().hfr_init()
    if check and st != HFR_OK:
        _raise(st)
    return st


def hfr_shutdown(check: bool = True) -> int:
    st = lib().hfr_shutdown()
    if check and st != HFR_OK:
        _raise(st)
    return st


def hfr_set_tuning(knob: int, value: int, check: bool = True) -> int:
    st = lib().hfr_set_tuning(int(knob), int(value))
    if check and st != HFR_OK:
        _raise(st)
    return st
