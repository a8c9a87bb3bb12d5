"""CPU oracle for the HFReduce reduction arithmetic (Algorithm 1 inner loop,
Algorithm 2 pass 1 of the paper).

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the
benchmark's ``cpu_baseline`` leg. The product (the HIP library and its Python
binding) never imports this package and this package never imports the product.

The arithmetic lives in ``hfr_oracle.cpp`` (plain single-threaded C++); this
module only compiles it with the host compiler and marshals numpy arrays.
bfloat16 and float16 buffers are numpy ``uint16`` arrays, fp8 buffers ``uint8`` arrays, holding the raw bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hfr_oracle.cpp")
_LIB = os.path.join(_HERE, "libhfr_oracle.so")

F32 = 0
BF16 = 1
F16 = 2
FP8_E4M3 = 3
FP8_E5M2 = 4
_NP_DTYPE = {F32: np.float32, BF16: np.uint16, F16: np.uint16, FP8_E4M3: np.uint8, FP8_E5M2: np.uint8}

# The flags are part of the oracle's definition: no contraction, no fast-math.
CXXFLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared"]

_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (host only). Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(["g++", *CXXFLAGS, "-o", tmp, _SRC], check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
            lib.oracle_reduce_sum.argtypes = [ctypes.POINTER(vp), ci, vp, sz, ci]
            lib.oracle_reduce_sum.restype = ci
            lib.oracle_combine_avg.argtypes = [vp, vp, vp, sz, ctypes.c_float, ci]
            lib.oracle_combine_avg.restype = ci
            lib.oracle_reduce_buckets.argtypes = [
                ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(sz), sz, ci, ci]
            lib.oracle_reduce_buckets.restype = ci
            lib.oracle_reduce_avg.argtypes = [ctypes.POINTER(vp), ci, vp, sz, ctypes.c_float, ci]
            lib.oracle_reduce_avg.restype = ci
            lib.oracle_slice_bounds.argtypes = [sz, ci, ci, ctypes.POINTER(sz), ctypes.POINTER(sz)]
            lib.oracle_slice_bounds.restype = None
            lib.oracle_reduce_scatter_slice.argtypes = [ctypes.POINTER(vp), ci, vp, sz, ci, ci, ci]
            lib.oracle_reduce_scatter_slice.restype = ci
            lib.oracle_broadcast.argtypes = [vp, ctypes.POINTER(vp), ci, sz, ci]
            lib.oracle_broadcast.restype = ci
            lib.oracle_narrow_bf16.argtypes = [vp, vp, sz]
            lib.oracle_narrow_bf16.restype = None
            lib.oracle_widen_bf16.argtypes = [vp, vp, sz]
            lib.oracle_widen_bf16.restype = None
            lib.oracle_narrow_fp8.argtypes = [vp, vp, sz, ci]
            lib.oracle_narrow_fp8.restype = None
            lib.oracle_widen_fp8.argtypes = [vp, vp, sz, ci]
            lib.oracle_widen_fp8.restype = None
            lib.oracle_narrow_f16.argtypes = [vp, vp, sz]
            lib.oracle_narrow_f16.restype = None
            lib.oracle_widen_f16.argtypes = [vp, vp, sz]
            lib.oracle_widen_f16.restype = None
            _lib = lib
    return _lib


def _check(arr: np.ndarray, dtype: int, n: int | None = None) -> np.ndarray:
    want = _NP_DTYPE[dtype]
    if arr.dtype != want or arr.ndim != 1 or not arr.flags.c_contiguous:
        raise ValueError("oracle buffers are 1-D contiguous %s arrays" % np.dtype(want).name)
    if n is not None and arr.shape[0] != n:
        raise ValueError("buffer length mismatch")
    return arr


def reduce_sum(ins, dtype: int, out: np.ndarray | None = None) -> np.ndarray:
    """Algorithm 1 inner loop: out = ((in0 + in1) + in2) + ... in fp32, index order.

    ``out`` may be one of ``ins`` (in-place form)."""
    lib = _load()
    K = len(ins)
    n = ins[0].shape[0]
    for a in ins:
        _check(a, dtype, n)
    if out is None:
        out = np.empty(n, dtype=_NP_DTYPE[dtype])
    _check(out, dtype, n)
    ptrs = (ctypes.c_void_p * K)(*[a.ctypes.data for a in ins])
    rc = lib.oracle_reduce_sum(ptrs, K, out.ctypes.data, n, dtype)
    if rc != 0:
        raise ValueError("oracle_reduce_sum rejected its arguments")
    return out


def combine_avg(a: np.ndarray, b: np.ndarray, scale, dtype: int,
                out: np.ndarray | None = None) -> np.ndarray:
    """Algorithm 2 pass 1 plus averaging: out = fl(fl(a + b) * scale) in fp32."""
    lib = _load()
    n = a.shape[0]
    _check(a, dtype, n)
    _check(b, dtype, n)
    if out is None:
        out = np.empty(n, dtype=_NP_DTYPE[dtype])
    _check(out, dtype, n)
    rc = lib.oracle_combine_avg(a.ctypes.data, b.ctypes.data, out.ctypes.data, n,
                                ctypes.c_float(float(np.float32(scale))), dtype)
    if rc != 0:
        raise ValueError("oracle_combine_avg rejected its arguments")
    return out


def reduce_buckets(buckets, dtype: int):
    """Algorithm 1's chunk loop over a bucket list.

    ``buckets`` is a list of (ins, out) pairs, ``ins`` a list of K arrays.
    Outputs are written in place and also returned as a list."""
    lib = _load()
    nb = len(buckets)
    if nb == 0:
        return []
    K = len(buckets[0][0])
    in_tab = (ctypes.c_void_p * (nb * K))()
    out_tab = (ctypes.c_void_p * nb)()
    n_tab = (ctypes.c_size_t * nb)()
    for bi, (ins, out) in enumerate(buckets):
        if len(ins) != K:
            raise ValueError("every bucket has K input buffers")
        n = out.shape[0]
        _check(out, dtype, n)
        for j, a in enumerate(ins):
            _check(a, dtype, n)
            in_tab[bi * K + j] = a.ctypes.data
        out_tab[bi] = out.ctypes.data
        n_tab[bi] = n
    rc = lib.oracle_reduce_buckets(in_tab, out_tab, n_tab, nb, K, dtype)
    if rc != 0:
        raise ValueError("oracle_reduce_buckets rejected its arguments")
    return [out for _, out in buckets]


def reduce_avg(ins, scale, dtype: int, out: np.ndarray | None = None) -> np.ndarray:
    """K-way in-order fp32 sum, one multiply by scale, one narrowing."""
    lib = _load()
    K = len(ins)
    n = ins[0].shape[0]
    for a in ins:
        _check(a, dtype, n)
    if out is None:
        out = np.empty(n, dtype=_NP_DTYPE[dtype])
    _check(out, dtype, n)
    ptrs = (ctypes.c_void_p * K)(*[a.ctypes.data for a in ins])
    rc = lib.oracle_reduce_avg(ptrs, K, out.ctypes.data, n, ctypes.c_float(float(np.float32(scale))), dtype)
    if rc != 0:
        raise ValueError("oracle_reduce_avg rejected its arguments")
    return out


def slice_bounds(n: int, rank: int, world: int):
    """[begin, end) of slice `rank` of `world` nearly equal slices of [0, n)."""
    lib = _load()
    b, e = ctypes.c_size_t(), ctypes.c_size_t()
    lib.oracle_slice_bounds(n, rank, world, ctypes.byref(b), ctypes.byref(e))
    return int(b.value), int(e.value)


def reduce_scatter_slice(ins, rank: int, world: int, dtype: int, out: np.ndarray) -> np.ndarray:
    """In-order K-way sum of slice `rank` only, written into `out` in place."""
    lib = _load()
    K = len(ins)
    n = ins[0].shape[0]
    for a in ins:
        _check(a, dtype, n)
    _check(out, dtype, n)
    ptrs = (ctypes.c_void_p * K)(*[a.ctypes.data for a in ins])
    rc = lib.oracle_reduce_scatter_slice(ptrs, K, out.ctypes.data, n, rank, world, dtype)
    if rc != 0:
        raise ValueError("oracle_reduce_scatter_slice rejected its arguments")
    return out


def broadcast(src: np.ndarray, K: int, dtype: int):
    """Algorithm 2 pass 2: K exact copies of src (returned as a list)."""
    lib = _load()
    n = src.shape[0]
    _check(src, dtype, n)
    outs = [np.empty(n, dtype=_NP_DTYPE[dtype]) for _ in range(K)]
    ptrs = (ctypes.c_void_p * max(K, 1))(*[o.ctypes.data for o in outs])
    rc = lib.oracle_broadcast(src.ctypes.data, ptrs, K, n, dtype)
    if rc != 0:
        raise ValueError("oracle_broadcast rejected its arguments")
    return outs


def narrow_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest even (test hook)."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape[0], dtype=np.uint16)
    lib.oracle_narrow_bf16(x.ctypes.data, out.ctypes.data, x.shape[0])
    return out


def widen_bf16(h: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> fp32, exact (test hook)."""
    lib = _load()
    h = np.ascontiguousarray(h, dtype=np.uint16)
    out = np.empty(h.shape[0], dtype=np.float32)
    lib.oracle_widen_bf16(h.ctypes.data, out.ctypes.data, h.shape[0])
    return out


def narrow_f16(x: np.ndarray) -> np.ndarray:
    """fp32 -> fp16 bit patterns, round to nearest even (test hook)."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape[0], dtype=np.uint16)
    lib.oracle_narrow_f16(x.ctypes.data, out.ctypes.data, x.shape[0])
    return out


def widen_f16(h: np.ndarray) -> np.ndarray:
    """fp16 bit patterns -> fp32, exact (test hook)."""
    lib = _load()
    h = np.ascontiguousarray(h, dtype=np.uint16)
    out = np.empty(h.shape[0], dtype=np.float32)
    lib.oracle_widen_f16(h.ctypes.data, out.ctypes.data, h.shape[0])
    return out


def narrow_fp8(x: np.ndarray, dtype: int) -> np.ndarray:
    """fp32 -> fp8 bit patterns (E4M3 or E5M2), round to nearest even (test hook)."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape[0], dtype=np.uint8)
    lib.oracle_narrow_fp8(x.ctypes.data, out.ctypes.data, x.shape[0], dtype)
    return out


def widen_fp8(b: np.ndarray, dtype: int) -> np.ndarray:
    """fp8 bit patterns -> fp32, exact (test hook)."""
    lib = _load()
    b = np.ascontiguousarray(b, dtype=np.uint8)
    out = np.empty(b.shape[0], dtype=np.float32)
    lib.oracle_widen_fp8(b.ctypes.data, out.ctypes.data, b.shape[0], dtype)
    return out
